// The fused polysemous scan (Section 3.3 two-step strategy; Section 4.2 "dual") for gfx950.
//
// One workgroup = one tile of TQ queries x one slice of the database.
//   * the TQ ADC tables (TQ * m * 256 float32) and the TQ running top-k lists live in LDS for
//     the lifetime of the workgroup;
//   * the TQ query codes live in scalar registers;
//   * every wave streams blocks of 64 x CB codes from memory into vector registers (16-byte
//     loads, four blocks per turn with the next four already requested; CB = 32 / TQ codes per
//     lane) and compares each code with all TQ query codes: xor + popcount-accumulate per
//     32-bit word, then one funnel shift that appends the "too far" bit to a 32-bit per-lane
//     mask (one bit per (code, query)): 5 integer instructions per (query, 64-bit code) pair;
//   * lanes that hold survivors append one (bit number, code position) entry per turn to a
//     per-wave queue in LDS, positions assigned with ballot + prefix popcount, so that the
//     expensive step runs on full wavefronts;
//   * whenever the queue holds 64 entries the wave scores the newest 64: re-reads the codes,
//     gathers m table entries each from LDS, sums them in float32 (j ascending) and compares
//     with the query's current bound on its k-th best distance;
//   * the few candidates that pass are spliced into the query's sorted list in LDS by the whole
//     wave, under a per-query lock (waves of the workgroup share the lists); workgroups of one
//     query tell each other how far their lists have come through a few words in global memory
//     (their k-th best distance, or -- a query cut into many slices -- an earlier entry of each
//     list, from which a bound on the k-th best of all of them follows: ScanArgs::pub_slots).
// Partial lists (one per query and slice) go to the workspace; a second kernel merges them.
//
// Ordering everywhere: (distance, id) ascending, lower id first on equal distance.
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "common.h"

namespace psc {
namespace {

constexpr int kQueueCap = 128;        // ring entries per wave (power of two, >= 2*64)
constexpr int kRelBits = 27;          // bits of a ring entry holding the position inside the slice
constexpr uint32_t kRelMask = (1u << kRelBits) - 1;
constexpr int64_t kMaxSliceLen = (int64_t)1 << kRelBits;
constexpr int kMfmaRelBits = 25;      // the same for the matrix-core filter (two more bits name the lane's row group)
constexpr uint32_t kMfmaRelMask = (1u << kMfmaRelBits) - 1;
constexpr int64_t kMfmaMaxSliceLen = (int64_t)1 << kMfmaRelBits;
constexpr int64_t kMfmaMinQueries = 9;  // fewer queries than this take the narrower xor/popcount tiles
constexpr int kMfmaTableBytes = 256 * 8;  // the bits-to-elements table of the matrix-core filter
constexpr int kSpinLimit = 1 << 22;   // bounded wait on a list lock (each turn sleeps)
constexpr int kManySlices = 4;        // slices per query from which the lists exchange more than their k-th best

struct IvfTile {
    int32_t job_begin, njobs, list, pad;
};

struct ScanArgs {
    const float *lut;         // [nq][M][256]
    const uint8_t *qcodes;    // [nq][M]
    const uint8_t *codes;     // [n][M]
    int64_t skip_first;       // >= 0: query q never returns database row skip_first + q (graph mode)
    int64_t nq, n;
    int64_t slice_len;
    int nslice;
    int64_t tiles_one;        // flat mode: the first tiles_one query tiles scan the whole database in one piece
    int k, kpad;
    uint32_t bias;            // 0x7fffffff - ht: bit 31 of (bias + distance) <=> distance > ht
    float *part_d;            // [nq][nslice][k]
    int64_t *part_i;          // [nq][nslice][k]
    int *status;              // set non-zero if a bounded wait expired
    // Per query, the smallest k-th-best distance any workgroup working for that query has
    // reached so far, as a sortable key (see dist_key).  Nothing farther than it can be in the
    // query's final top-k, so every workgroup of the query prunes with it: the partial lists
    // of one query behave like one stream instead of one warm-up per slice or list.
    uint32_t *gthr;           // [number of queries][pub_slots] (pub_slots = 1: as described; more: see pub_slots)
    const int32_t *job_q;     // inverted-file mode: query of each job (index into gthr)
    // inverted-file mode (Section 4.3): a tile = up to TQ (query, list) jobs of ONE list, rows
    // job_begin.. of the job-sorted tables / query codes; the scanned range is that list
    const IvfTile *tiles;     // [*ntiles]
    const int *ntiles;        // device-side count (the grid is an upper bound)
    const int64_t *list_off;  // [nlist+1] list boundaries in `codes`
    const int32_t *ext_ids;   // [n] id of each stored code
    const int32_t *job_slot;  // [njobs] partial list (query * nprobe + probe) a job writes
    // Residual tables of the inverted file, not stored per job.  With o the mean coarse
    // centroid, q~ = q - o and g~ = g - o for the coarse centroid g of the tile's list,
    //   ||(q - g)_j - c||^2 = (||c||^2 - 2 q~_j . c)  +  2 g~_j . c  +  ||(q - g)_j||^2
    //                       = lut[query][j][c] + list_tab[list][j][c] + (one number per job and j),
    // which a tile puts together in LDS (the first two, whose sum ||c||^2 - 2 (q - g)_j . c is of
    // the size of the result, before the third).  The query code of a job is the arg-min of those
    // rows.  list_tab == nullptr: `lut` holds one finished table per job, in job order (indexes
    // whose coarse centroids lie so far apart that the sum above would lose too many bits).
    const float *list_tab;    // [nlist][M][256]
    const float *queries;     // [nq][dim] raw query vectors
    const float *coarse;      // [nlist + 1][dim] coarse centroids, then their mean
    uint8_t *job_qcodes;      // [njobs][M] out: query code of each job
    int dim, nlist;
    // A few jobs, one per tile (latency matters): the tile's unused query slots serve the same
    // job, each wave feeding the list of slot wave % TQ, so that a list's lock is shared by a
    // quarter of the waves while the lists fill; the lists are merged when the tile ends.
    int spread_lists = 0;
    // Many slices per query (a handful of queries over a large database: every slice's list
    // would otherwise warm up on its own share only).  gthr then holds pub_slots words per query;
    // a list with pub_r entries or more keeps the key of its pub_r-th best in word slice %
    // pub_slots (atomic minimum over the lists that share the word).  Lists of different words
    // hold different codes, so a value v with pub_kth words at or below it has pub_kth * pub_r
    // >= k codes at or below it: nothing farther than v is in the query's top k.  With one word,
    // pub_r = k and pub_kth = 1 this is the plain exchange of k-th best distances.
    int pub_slots = 1, pub_r = 0, pub_kth = 1;
};

// Flat mode: which queries and which part of the database a workgroup works on.  Query tiles
// 0 .. tiles_one-1 are scanned in one piece each (they fill whole rounds of workgroups that run
// together); the tiles after them are cut into nslice slices each, so that the last, partial
// round finishes in 1/nslice of the time instead of leaving compute units idle.  A query scanned
// in one piece builds one list instead of nslice: fewer insertions and a cheaper merge.
struct FlatTile {
    int slice;
    bool whole;  // one piece: the other slices' places in the partial lists get padding
    int64_t q0, slice_begin, slice_end;
};
__device__ __forceinline__ FlatTile flat_tile(const ScanArgs &a, int64_t tile, int tq)
{
    FlatTile t;
    if (tile < a.tiles_one) {
        t.slice = 0;
        t.whole = true;
        t.q0 = tile * tq;
        t.slice_begin = 0;
        t.slice_end = a.n;
    } else {
        const int64_t u = tile - a.tiles_one;
        t.slice = (int)(u % a.nslice);
        t.whole = false;
        t.q0 = (a.tiles_one + u / a.nslice) * tq;
        t.slice_begin = (int64_t)t.slice * a.slice_len;
        t.slice_end = (t.slice_begin + a.slice_len) < a.n ? (t.slice_begin + a.slice_len) : a.n;
    }
    return t;
}
// Padding for the partial lists a one-piece tile leaves unused (slices 1 .. nslice-1 of its queries).
__device__ __forceinline__ void pad_unused_slices(const ScanArgs &a, int64_t q0, int nvq, int tid, int nthreads)
{
    const int per_q = (a.nslice - 1) * a.k;
    for (int e = tid; e < nvq * per_q; e += nthreads) {
        const int q = e / per_q, r = e - q * per_q;
        const int64_t o = ((q0 + q) * a.nslice + 1) * a.k + r;
        a.part_d[o] = __builtin_inff();
        a.part_i[o] = (int64_t)-1;
    }
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

__device__ __forceinline__ int prefix_count(uint64_t mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                          __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ float bcast_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ uint32_t bcast_u(uint32_t v, int lane)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

// Shared-memory view of one workgroup.  The pointers carry the LDS address space explicitly so
// that every access is a ds_* instruction.
#define PSC_LDS __attribute__((address_space(3)))
typedef PSC_LDS float lds_f32;
typedef PSC_LDS volatile float lds_vf32;
typedef PSC_LDS volatile uint32_t lds_vu32;
typedef PSC_LDS uint32_t lds_u32;
typedef PSC_LDS volatile int lds_vi32;
typedef PSC_LDS int lds_i32;

typedef PSC_LDS volatile uint64_t lds_vu64;

// One list entry = (sortable distance key, id) packed in 64 bits, key in the high word, so that
// the unsigned 64-bit order is the (distance, id) order.  The key is the usual order-preserving
// map of float bits to unsigned (negative values flip all bits, others flip the sign bit);
// -0 is folded into +0 first so that equal distances get equal keys.
__device__ __forceinline__ uint32_t dist_key(float d)
{
    const uint32_t u = __float_as_uint(d + 0.0f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_dist(uint32_t key)
{
    return __uint_as_float(key ^ ((key >> 31) ? 0x80000000u : 0xffffffffu));
}
constexpr uint32_t kKeyInf = 0xff800000u;  // dist_key(+infinity)
__device__ __forceinline__ uint64_t pack_entry(float d, uint32_t id)
{
    return ((uint64_t)dist_key(d) << 32) | id;
}
__device__ __forceinline__ float entry_dist(uint64_t e) { return key_dist((uint32_t)(e >> 32)); }
__device__ __forceinline__ uint32_t entry_id(uint64_t e) { return (uint32_t)e; }

template <int M, int TQ>
struct Lds {
    lds_f32 *lut;    // [TQ][M][256]
    lds_vu64 *top;   // [TQ][kpad] sorted ascending
    lds_vf32 *thr;   // [TQ] bound on the query's k-th best distance (+inf while nothing is known)
    lds_i32 *lock;   // [TQ] number of entries in the list, or kLocked while a wave works on it
    lds_i32 *gidx;   // [TQ] the slot's query as an index into the shared thresholds (-1: empty slot)
    lds_i32 *pslot;  // [TQ] word of the query's shared thresholds the slot's list publishes to
    lds_f32 *sterm;  // [TQ][M] inverted file: the per-job, per-sub-quantizer constant of the tables
    lds_u32 *qcw;    // [TQ][M/4] inverted file: the jobs' query codes
    lds_u32 *queue;  // [nwaves][kQueueCap]; private to a wave: LDS keeps a wave's accesses in order
    lds_u32 *dump;   // [nwaves][64] where lanes with nothing to queue write
    __device__ __forceinline__ Lds(PSC_LDS unsigned char *base, int kpad, int nwaves)
    {
        lut = (lds_f32 *)base;
        top = (lds_vu64 *)(lut + TQ * M * 256);
        thr = (lds_vf32 *)(top + TQ * kpad);
        lock = (lds_i32 *)(thr + TQ);
        gidx = lock + TQ;
        pslot = gidx + TQ;
        sterm = (lds_f32 *)(pslot + TQ);
        qcw = (lds_u32 *)(sterm + TQ * M);
        queue = qcw + TQ * M / 4;
        dump = queue + nwaves * kQueueCap;
    }
};

// ---- the Hamming test of Section 3.3, hand-written ------------------------------------------
// For one code (words w) and NQ queries whose code words sit in scalar registers: per pair one
// v_xor and one v_bcnt (population count plus accumulator) per 32-bit word, the accumulator
// starting at `bias` = 0x7fffffff - ht so that its sign bit says "farther than ht", and one
// v_alignbit that shifts that bit into `far`.  5 instructions per 64-bit pair, 9 per 128-bit
// pair; written out because the compiler, left to itself, sometimes regroups the sum into
// (count + count) + bias at the price of one more instruction per pair.
#define PSC_PAIR_W2(QA, QB)                          \
    "v_xor_b32_e32 %[t0], %[" QA "], %[w0]\n\t"       \
    "v_bcnt_u32_b32 %[t0], %[t0], %[b]\n\t"           \
    "v_xor_b32_e32 %[t1], %[" QB "], %[w1]\n\t"       \
    "v_bcnt_u32_b32 %[t0], %[t1], %[t0]\n\t"          \
    "v_alignbit_b32 %[far], %[far], %[t0], 31\n\t"
#define PSC_PAIR_W4(QA, QB, QC, QD)                  \
    "v_xor_b32_e32 %[t0], %[" QA "], %[w0]\n\t"       \
    "v_bcnt_u32_b32 %[t0], %[t0], %[b]\n\t"           \
    "v_xor_b32_e32 %[t1], %[" QB "], %[w1]\n\t"       \
    "v_bcnt_u32_b32 %[t0], %[t1], %[t0]\n\t"          \
    "v_xor_b32_e32 %[t1], %[" QC "], %[w2]\n\t"       \
    "v_bcnt_u32_b32 %[t0], %[t1], %[t0]\n\t"          \
    "v_xor_b32_e32 %[t1], %[" QD "], %[w3]\n\t"       \
    "v_bcnt_u32_b32 %[t0], %[t1], %[t0]\n\t"          \
    "v_alignbit_b32 %[far], %[far], %[t0], 31\n\t"

// four queries, 64-bit codes
__device__ __forceinline__ void hamming_test4(uint32_t &far, const uint32_t (&w)[2], uint32_t bias,
                                              const uint32_t (*q)[2])
{
    uint32_t t0, t1;
    asm(PSC_PAIR_W2("q0a", "q0b") PSC_PAIR_W2("q1a", "q1b") PSC_PAIR_W2("q2a", "q2b") PSC_PAIR_W2("q3a", "q3b")
        : [far] "+v"(far), [t0] "=&v"(t0), [t1] "=&v"(t1)
        : [w0] "v"(w[0]), [w1] "v"(w[1]), [b] "s"(bias), [q0a] "s"(q[0][0]), [q0b] "s"(q[0][1]),
          [q1a] "s"(q[1][0]), [q1b] "s"(q[1][1]), [q2a] "s"(q[2][0]), [q2b] "s"(q[2][1]), [q3a] "s"(q[3][0]),
          [q3b] "s"(q[3][1]));
}
// eight queries, 64-bit codes
__device__ __forceinline__ void hamming_test8(uint32_t &far, const uint32_t (&w)[2], uint32_t bias,
                                              const uint32_t (*q)[2])
{
    uint32_t t0, t1;
    asm(PSC_PAIR_W2("q0a", "q0b") PSC_PAIR_W2("q1a", "q1b") PSC_PAIR_W2("q2a", "q2b") PSC_PAIR_W2("q3a", "q3b")
            PSC_PAIR_W2("q4a", "q4b") PSC_PAIR_W2("q5a", "q5b") PSC_PAIR_W2("q6a", "q6b") PSC_PAIR_W2("q7a", "q7b")
        : [far] "+v"(far), [t0] "=&v"(t0), [t1] "=&v"(t1)
        : [w0] "v"(w[0]), [w1] "v"(w[1]), [b] "s"(bias), [q0a] "s"(q[0][0]), [q0b] "s"(q[0][1]),
          [q1a] "s"(q[1][0]), [q1b] "s"(q[1][1]), [q2a] "s"(q[2][0]), [q2b] "s"(q[2][1]), [q3a] "s"(q[3][0]),
          [q3b] "s"(q[3][1]), [q4a] "s"(q[4][0]), [q4b] "s"(q[4][1]), [q5a] "s"(q[5][0]), [q5b] "s"(q[5][1]),
          [q6a] "s"(q[6][0]), [q6b] "s"(q[6][1]), [q7a] "s"(q[7][0]), [q7b] "s"(q[7][1]));
}
// four queries, 128-bit codes
__device__ __forceinline__ void hamming_test4(uint32_t &far, const uint32_t (&w)[4], uint32_t bias,
                                              const uint32_t (*q)[4])
{
    uint32_t t0, t1;
    asm(PSC_PAIR_W4("q0a", "q0b", "q0c", "q0d") PSC_PAIR_W4("q1a", "q1b", "q1c", "q1d")
            PSC_PAIR_W4("q2a", "q2b", "q2c", "q2d") PSC_PAIR_W4("q3a", "q3b", "q3c", "q3d")
        : [far] "+v"(far), [t0] "=&v"(t0), [t1] "=&v"(t1)
        : [w0] "v"(w[0]), [w1] "v"(w[1]), [w2] "v"(w[2]), [w3] "v"(w[3]), [b] "s"(bias), [q0a] "s"(q[0][0]),
          [q0b] "s"(q[0][1]), [q0c] "s"(q[0][2]), [q0d] "s"(q[0][3]), [q1a] "s"(q[1][0]), [q1b] "s"(q[1][1]),
          [q1c] "s"(q[1][2]), [q1d] "s"(q[1][3]), [q2a] "s"(q[2][0]), [q2b] "s"(q[2][1]), [q2c] "s"(q[2][2]),
          [q2d] "s"(q[2][3]), [q3a] "s"(q[3][0]), [q3b] "s"(q[3][1]), [q3c] "s"(q[3][2]), [q3d] "s"(q[3][3]));
}
// all TQ queries of a tile against one code
template <int TQ, int WPC>
__device__ __forceinline__ void hamming_test_tile(uint32_t &far, const uint32_t (&w)[WPC], uint32_t bias,
                                                  const uint32_t (&qw)[TQ][WPC])
{
    if constexpr (WPC == 2 && TQ % 8 == 0) {
#pragma unroll
        for (int q = 0; q < TQ; q += 8) hamming_test8(far, w, bias, &qw[q]);
    } else {
#pragma unroll
        for (int q = 0; q < TQ; q += 4) hamming_test4(far, w, bias, &qw[q]);
    }
}

// Smallest value of v over the wave, in every lane: four row-local steps on the data-parallel
// path, then the four row results through scalar registers.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    auto step = [](uint32_t x, uint32_t y) { return y < x ? y : x; };
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xf, 0xf, false));   // lane ^ 1
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xf, 0xf, false));   // lane ^ 2
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xf, 0xf, false));  // mirror in 8
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xf, 0xf, false));  // mirror in 16
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
    const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return step(step(r0, r1), step(r2, r3));
}

constexpr int kLocked = -1;

// The 64-bit value held by the lane below (lane 0 receives `first`): a whole-wave shift by one
// lane on the data-parallel path.
__device__ __forceinline__ uint64_t from_lane_below(uint64_t v, uint64_t first)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)first, (int)(uint32_t)v, 0x138, 0xf,
                                                              0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(first >> 32), (int)(uint32_t)(v >> 32),
                                                              0x138, 0xf, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t lane_value_u64(uint64_t v, int l)
{
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l) << 32) |
           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
}
// Lower a threshold in LDS, no answer awaited.
__device__ __forceinline__ void lower_threshold(lds_vf32 *p, float v)
{
    (void)__hip_atomic_fetch_min((lds_f32 *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// An upper bound on the kth smallest (kth >= 1) of the keys held by the 64 lanes, the same in
// every lane: the key's upper 20 bits are found one by one, by counting the lanes at or below
// the value tried (sign, exponent and 11 bits of mantissa: within 0.05% of the exact value),
// the rest is filled with ones.  kKeyInf or above: fewer than kth lanes hold a finite key.
__device__ __forceinline__ uint32_t wave_kth_smallest_bound(uint32_t v, int kth)
{
    uint32_t prefix = 0u;
#pragma unroll 1
    for (int bit = 31; bit >= 12; --bit) {
        const uint32_t trial = prefix | ((1u << bit) - 1u);
        if (__builtin_popcountll(ballot64(v <= trial)) < kth) prefix |= 1u << bit;
    }
    return prefix | 0xfffu;
}

// Insert the candidates held by the lanes in `mine` (all for query slot q) into q's sorted list.
// Executed by the whole wave; mine is wave-uniform.  The slot's lock word doubles as the entry
// count, so taking the lock also fetches the count and releasing it stores the new one.
// Lists of up to 128 entries (two per lane) are read into registers once, every candidate is
// ranked by ballot and spliced in with a one-lane shift, and the list is written back once: two
// trips to LDS per call however many candidates it brings.
// SHARE: the list's k-th best is published to the other workgroups of the query.  EAGER: every
// call also reads what they have published (worth the wait at its end when a query is spread
// over hundreds of workgroups; with the few dozen lists of an inverted-file probe the reads made
// once per batch of candidates are enough).
template <int M, int TQ, bool SHARE, bool EAGER>
__device__ __forceinline__ void insert_candidates(const Lds<M, TQ> &s, const ScanArgs &a, int q, uint64_t mine,
                                                  float d, uint32_t id)
{
    const int lane = lane_id();
    // The other waves of the SIMD are busy filtering and would get three of every four issue
    // slots: whoever works on a list (and may hold its lock) goes first.
    __builtin_amdgcn_s_setprio(3);
    int cnt = kLocked;
    if (lane == 0) {
        int spins = 0;
        while (true) {
            cnt = __hip_atomic_exchange(&s.lock[q], kLocked, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (cnt != kLocked || ++spins > kSpinLimit) break;
            __builtin_amdgcn_s_sleep(2);
        }
    }
    cnt = __builtin_amdgcn_readfirstlane(cnt);
    if (cnt == kLocked) {  // never expected: flag the run instead of waiting for ever
        if (lane == 0) atomicExch(a.status, 1);
        __builtin_amdgcn_s_setprio(0);
        return;
    }
    // Everything the lock protects lives in LDS, which serves the accesses of a wave in the order
    // they were issued and those of different waves one after the other: a lock word taken by
    // an exchange and given back by a plain store after the data needs no hardware fence.  (A
    // workgroup-scope fence would also wait for every global load the wave has in flight, its
    // prefetched codes included, with the lock held.)  Only the compiler must keep the order.
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    // What the other workgroups of this query have reached by now: asked for here, used after
    // the lock is given back, so the trip to memory overlaps the work on the list.
    uint32_t seen = kKeyInf;
    int gi = -1;
    const bool many = SHARE && a.pub_slots > 1;  // (wave-uniform) the exchange over many slices
    uint32_t slots_seen = kKeyInf;               // many: lane l holds word l of the query
    int my_slot = 0;                             // many: the word this list publishes to
    if constexpr (SHARE) {
        if (many) {
            gi = __builtin_amdgcn_readfirstlane(s.gidx[q]);
            my_slot = __builtin_amdgcn_readfirstlane(s.pslot[q]);
            if (lane < a.pub_slots)
                slots_seen = __hip_atomic_load(&a.gthr[(int64_t)gi * a.pub_slots + lane], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
        } else if (lane == 0) {
            gi = s.gidx[q];
            if constexpr (EAGER) seen = __hip_atomic_load(&a.gthr[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    lds_vu64 *list = s.top + q * a.kpad;
    const int k = a.k;
    const int pr = a.pub_r;      // (1 <= pub_r <= k whenever `many`)
    uint32_t own_key = kKeyInf;  // the list's k-th best once it is full
    uint32_t pub_key = kKeyInf;  // many: the list's pub_r-th best once it has that many entries
    bool changed = false;
    float thr_old;
    if (k <= 128) {
        const int i0 = lane, i1 = 64 + lane;  // the two list places of the lane
        thr_old = s.thr[q];
        mine &= ballot64(d <= thr_old);  // the threshold may have dropped since the candidates were scored
        // Short lists (k <= 64, or a list that stays within 64 entries after this call: most lists
        // of inverted-file jobs) live in one register per lane.
        const bool one = k <= 64 || cnt + __builtin_popcountll(mine) <= 64;  // (wave-uniform)
        uint64_t e0 = ~0ull, e1 = ~0ull;  // places past the end hold the largest key
        if (i0 < cnt) e0 = list[i0];
        if (one) {
            while (mine) {
                const int src = __builtin_ctzll(mine);
                mine &= mine - 1;
                const uint64_t cand = pack_entry(bcast_f(d, src), bcast_u(id, src));
                const int pos = __builtin_popcountll(ballot64(e0 < cand));
                if (pos >= k) continue;
                const uint64_t up0 = from_lane_below(e0, e0);
                e0 = i0 > pos ? up0 : (i0 == pos ? cand : e0);
                if (i0 >= k) e0 = ~0ull;
                if (cnt < k) ++cnt;
                changed = true;
            }
            if (changed) {
                if (i0 < cnt) list[i0] = e0;
                if (cnt == k) own_key = (uint32_t)(lane_value_u64(e0, (k - 1) & 63) >> 32);  // (k <= 64 here)
                if (many && cnt >= pr) pub_key = (uint32_t)(lane_value_u64(e0, (pr - 1) & 63) >> 32);  // (pr <= cnt <= 64)
            }
        } else {
            if (i1 < cnt) e1 = list[i1];
            while (mine) {
                const int src = __builtin_ctzll(mine);
                mine &= mine - 1;
                const uint64_t cand = pack_entry(bcast_f(d, src), bcast_u(id, src));
                const int pos = __builtin_popcountll(ballot64(e0 < cand)) + __builtin_popcountll(ballot64(e1 < cand));
                if (pos >= k) continue;
                // places pos.. move one down the list; what falls off the end is forgotten
                const uint64_t up0 = from_lane_below(e0, e0);
                const uint64_t up1 = from_lane_below(e1, lane_value_u64(e0, 63));
                e0 = i0 > pos ? up0 : (i0 == pos ? cand : e0);
                e1 = i1 > pos ? up1 : (i1 == pos ? cand : e1);
                if (i0 >= k) e0 = ~0ull;
                if (i1 >= k) e1 = ~0ull;
                if (cnt < k) ++cnt;
                changed = true;
            }
            if (changed) {
                if (i0 < cnt) list[i0] = e0;
                if (i1 < cnt) list[i1] = e1;
                if (cnt == k) own_key = (uint32_t)(lane_value_u64(k <= 64 ? e0 : e1, (k - 1) & 63) >> 32);
                if (many && cnt >= pr) pub_key = (uint32_t)(lane_value_u64(pr <= 64 ? e0 : e1, (pr - 1) & 63) >> 32);
            }
        }
    } else {
        thr_old = s.thr[q];
        while (mine) {
            const int src = __builtin_ctzll(mine);
            mine &= mine - 1;
            const uint64_t cand = pack_entry(bcast_f(d, src), bcast_u(id, src));
            if (cnt == k && !(cand < list[k - 1])) continue;
            // entries pos..last-1 move one place down the list (the k-th falls off when full)
            const int last = cnt < k ? cnt : k - 1;
            int pos = 0;
            for (int base = 0; base < cnt; base += 64) {
                const int p = base + lane;
                const bool before = p < cnt && list[p] < cand;
                pos += __builtin_popcountll(ballot64(before));
            }
            if (last > pos) {
                for (int base = ((last - 1) >> 6) << 6; base >= ((pos >> 6) << 6); base -= 64) {
                    const int p = base + lane;
                    const bool mv = p >= pos && p < last;
                    uint64_t e = 0;
                    if (mv) e = list[p];
                    __builtin_amdgcn_wave_barrier();
                    if (mv) list[p + 1] = e;
                    __builtin_amdgcn_wave_barrier();
                }
            }
            if (lane == 0) list[pos] = cand;
            if (cnt < k) ++cnt;
            changed = true;
            __builtin_amdgcn_wave_barrier();
        }
        if (changed && cnt == k) own_key = (uint32_t)(list[k - 1] >> 32);
        if (changed && many && cnt >= pr) pub_key = (uint32_t)(list[pr - 1] >> 32);
    }
    const float own = key_dist(own_key);
    const bool lowered = own < thr_old;  // this list's k-th best is below everything known so far
    if (lowered && lane == 0) lower_threshold(&s.thr[q], own);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    if (lane == 0) {
        __hip_atomic_store(&s.lock[q], cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        // Outside the lock: adopt what the others had reached, and tell them (no answer awaited).
        if constexpr (SHARE) {
            if (!many) {
                if (seen != kKeyInf && key_dist(seen) < (lowered ? own : thr_old))
                    lower_threshold(&s.thr[q], key_dist(seen));
                if (lowered && own_key < seen)
                    (void)__hip_atomic_fetch_min(&a.gthr[gi], own_key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    if constexpr (SHARE) {
        if (many) {
            // the word of this list first (as read at the start, or what the list has just reached)
            if (lane == my_slot) {
                if (pub_key < slots_seen) {
                    slots_seen = pub_key;
                    (void)__hip_atomic_fetch_min(&a.gthr[(int64_t)gi * a.pub_slots + lane], pub_key, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            const uint32_t bound = wave_kth_smallest_bound(slots_seen, a.pub_kth);
            if (lane == 0 && bound < kKeyInf && key_dist(bound) < (lowered ? own : thr_old))
                lower_threshold(&s.thr[q], key_dist(bound));
        }
    }
    __builtin_amdgcn_s_setprio(0);
}

// What the other workgroups of the tile's queries have reached.  `ask`: lane q < TQ requests the
// shared threshold of slot q.  `adopt`: lowers the slots' own thresholds to the answers.  Callers
// ask where a batch of candidates starts, next to a memory access of their own that they wait
// for anyway, and adopt before the candidates are tested -- but only while lists are changing
// (the previous batch inserted something), so that a settled scan asks nothing.
template <int M, int TQ>
__device__ __forceinline__ uint32_t ask_shared_thresholds(const Lds<M, TQ> &s, const ScanArgs &a)
{
    const int lane = lane_id();
    uint32_t g = kKeyInf;
    if (a.pub_slots > 1) return g;  // (the exchange over many slices happens where lists change)
    if (lane < TQ) {
        const int gi = s.gidx[lane];
        if (gi >= 0) g = __hip_atomic_load(&a.gthr[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return g;
}
template <int M, int TQ>
__device__ __forceinline__ void adopt_shared_thresholds(const Lds<M, TQ> &s, uint32_t g)
{
    const int lane = lane_id();
    if (lane < TQ && g != kKeyInf) lower_threshold(&s.thr[lane], key_dist(g));
}

// Inverted-file tiles start at different times: a job whose query has been served by other lists
// already starts from what those have published (ScanArgs::pub_slots) instead of +infinity.
// Wave w takes job slot w; called after the barrier that follows the per-slot state.
template <int M, int TQ>
__device__ __forceinline__ void start_from_published_bounds(const Lds<M, TQ> &s, const ScanArgs &a, int wave, int nvq)
{
    if (a.pub_slots <= 1 || wave >= nvq) return;
    const int lane = lane_id();
    const int gi = __builtin_amdgcn_readfirstlane(s.gidx[wave]);
    uint32_t v = kKeyInf;
    if (lane < a.pub_slots)
        v = __hip_atomic_load(&a.gthr[(int64_t)gi * a.pub_slots + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ballot64(v != kKeyInf) == 0) return;  // (nothing published yet)
    const uint32_t bound = wave_kth_smallest_bound(v, a.pub_kth);
    if (lane == 0 && bound < kKeyInf) lower_threshold(&s.thr[wave], key_dist(bound));
}

// State a wave carries from one batch of candidates to the next for the exchange above.
struct SharedAsk {
    bool wanted = true;  // wave-uniform: the previous batch changed a list (or there was none yet)
};

// The queueing loop of the fused kernels, hand-scheduled (see the comment where it is used).
// Operands: sv (survivor bits of the lane, consumed), fill (entries waiting, scalar), base (byte
// address of queue slot `fill`, scalar), rel0 (low bits of the lane's entries), dump (address a
// lane without a bit writes to); t0, t1 vector and n scalar temporaries.
#define PSC_QUEUE_TURNS                                    \
    "1:\n\t"                                               \
    "v_cmp_ne_u32_e32 vcc, 0, %[sv]\n\t"                   \
    "s_cbranch_vccz 2f\n\t"                                \
    "v_mbcnt_lo_u32_b32 %[t0], vcc_lo, 0\n\t"              \
    "v_mbcnt_hi_u32_b32 %[t0], vcc_hi, %[t0]\n\t"          \
    "v_ffbl_b32_e32 %[t1], %[sv]\n\t"                      \
    "v_lshl_add_u32 %[t0], %[t0], 2, %[base]\n\t"          \
    "v_lshl_or_b32 %[t1], %[t1], 27, %[rel0]\n\t"          \
    "v_cndmask_b32_e32 %[t0], %[dump], %[t0], vcc\n\t"     \
    "ds_write_b32 %[t0], %[t1]\n\t"                        \
    "s_bcnt1_i32_b64 %[n], vcc\n\t"                        \
    "v_add_u32_e32 %[t0], -1, %[sv]\n\t"                   \
    "s_lshl2_add_u32 %[base], %[n], %[base]\n\t"           \
    "v_and_b32_e32 %[sv], %[sv], %[t0]\n\t"                \
    "s_add_i32 %[fill], %[fill], %[n]\n\t"                 \
    "s_cmp_lt_i32 %[fill], 64\n\t"                         \
    "s_cbranch_scc1 1b\n\t"                                \
    "2:"

// Score `nvalid` (<= 64) entries of the wave's queue, starting at `ring`, and feed the ones that
// beat the current threshold to the lists.  `slice_codes` = the codes of the tile's slice
// (position 0 of the entries); `self0 + q` = the position query slot q must not return (graph
// mode; a value no position can take otherwise).
// MFMA_BITS: the entries come from the matrix-core filter (see scan_mfma_kernel for their layout).
template <int M, int TQ, bool IVF, bool SHARE, bool MFMA_BITS = false>
__device__ __forceinline__ void drain(const Lds<M, TQ> &s, const ScanArgs &a, const lds_u32 *ring, int nvalid,
                                      const uint8_t *slice_codes, int64_t slice_begin, uint32_t self0,
                                      SharedAsk &ask)
{
    const int lane = lane_id();
    const bool act = lane < nvalid;
    float d = __builtin_inff();
    float thr = -__builtin_inff();
    uint32_t rel = 0;
    int q = 0;
    uint32_t shared = kKeyInf;
    if constexpr (SHARE) {
        if (ask.wanted) shared = ask_shared_thresholds<M, TQ>(s, a);
    }
    if (act) {
        // entry = (b << kRelBits) | position of the lane's first code; b = c * TQ + (TQ - 1 - q)
        const uint32_t e = ring[lane];
        if constexpr (MFMA_BITS) {
            const uint32_t idx = ~e >> kRelBits;  // 31 - (bit number): 4 * (16-code group) + row
            q = (int)(4u * ((e >> kMfmaRelBits) & 3u) + (idx & 3u));
            rel = (e & kMfmaRelMask) + 16u * (idx >> 2);
        } else {
            const uint32_t b = e >> kRelBits;
            q = (int)((TQ - 1) - (b & (TQ - 1)));
            rel = (e & kRelMask) + b / TQ;
        }
        const uint32_t *cw = (const uint32_t *)(slice_codes + (uint64_t)rel * M);
        uint32_t w[M / 4];
        if constexpr (M == 8) {
            const uint2 v = *(const uint2 *)cw;
            w[0] = v.x;
            w[1] = v.y;
        } else {
            const uint4 v = *(const uint4 *)cw;
            w[0] = v.x;
            w[1] = v.y;
            w[2] = v.z;
            w[3] = v.w;
        }
        if constexpr (SHARE) {
            if (ask.wanted) adopt_shared_thresholds<M, TQ>(s, shared);
        }
        // The gathers are issued last sub-quantizer first and summed first sub-quantizer first:
        // LDS answers in order, so the first addition waits for all of them and the others for
        // nothing (one wait instruction instead of one per addition).
        const lds_f32 *t = s.lut + q * (M * 256);
        thr = s.thr[q];
        if constexpr (IVF) {
            float tv[M];
#pragma unroll
            for (int j = M - 1; j >= 0; --j) {
                const uint32_t byte = (w[j >> 2] >> (8 * (j & 3))) & 0xffu;
                tv[j] = t[j * 256 + byte];
            }
            float acc = tv[0];
#pragma unroll
            for (int j = 1; j < M; ++j) acc += tv[j];
            d = acc;
        } else {
            // Tables of squared distances have no negative entries, so the sum over the first
            // sub-quantizers already bounds the distance from below: once the lists are warm it
            // rejects nearly every survivor, and the other gathers are issued only if some lane
            // of the wave still needs them.  The additions keep their order (j ascending), so a
            // distance that is finished is the same float32 as without the shortcut.
            constexpr int M0 = (M * 3) / 8;
            float tv[M];
#pragma unroll
            for (int j = M0 - 1; j >= 0; --j) {
                const uint32_t byte = (w[j >> 2] >> (8 * (j & 3))) & 0xffu;
                tv[j] = t[j * 256 + byte];
            }
            float acc = tv[0];
#pragma unroll
            for (int j = 1; j < M0; ++j) acc += tv[j];
            if (acc <= thr) {
#pragma unroll
                for (int j = M - 1; j >= M0; --j) {
                    const uint32_t byte = (w[j >> 2] >> (8 * (j & 3))) & 0xffu;
                    tv[j] = t[j * 256 + byte];
                }
#pragma unroll
                for (int j = M0; j < M; ++j) acc += tv[j];
                d = acc;
            }
        }
    } else {
        if constexpr (SHARE) {
            if (ask.wanted) adopt_shared_thresholds<M, TQ>(s, shared);
        }
    }
    bool pass = d <= thr;  // (lanes without an entry: +inf <= -inf)
    uint32_t key = rel;    // what breaks distance ties: the position, or the stored id
    if constexpr (IVF) {
        if (pass) key = (uint32_t)a.ext_ids[slice_begin + rel];
    } else {
        pass = pass && rel != self0 + (uint32_t)q;  // a vector is not its own neighbour
    }
    uint64_t pm = ballot64(pass);
    ask.wanted = pm != 0;
    while (pm) {
        const int leader = __builtin_ctzll(pm);
        const int qcur = __builtin_amdgcn_readlane(q, leader);
        const uint64_t mine = ballot64(pass && q == qcur);
        pm &= ~mine;
        insert_candidates<M, TQ, SHARE, SHARE && !IVF>(s, a, qcur, mine, d, key);
    }
}

// Inverted-file tile set-up, shared by the fused kernels: the residual tables of the tile's jobs
// put together in LDS (see ScanArgs::list_tab) and the jobs' query codes taken from them (s.qcw).
// Called by the whole workgroup (NW waves) after the per-slot state (s.gidx) is written; ends with
// a barrier.
template <int M, int TQ, int NW>
__device__ __forceinline__ void stage_list_tables(const Lds<M, TQ> &s, const ScanArgs &a, int tile_list, int64_t q0,
                                                  int nvq)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int dsub = a.dim / M;
    // direct: the jobs' tables were built one by one by direct differences (a.lut holds them in job
    // order); nothing to put together
    const bool direct = a.list_tab == nullptr;
    if (!direct) {
        // the list's centroid and the jobs' queries staged where the tables will go (all loads of the
        // workgroup in flight together; (TQ + 1) * dim floats fit: dim <= 1024 = a quarter of one
        // job's tables at M = 8)
        PSC_LDS float *gs = (PSC_LDS float *)s.lut, *xs = gs + a.dim;
        for (int e = tid; e < (nvq + 1) * a.dim; e += NW * 64) {
            const int q = e / a.dim - 1, t = e % a.dim;
            const float *row = q < 0 ? a.coarse + (int64_t)tile_list * a.dim
                                     : a.queries + (int64_t)a.job_q[q0 + q] * a.dim;
            gs[e] = row[t];
        }
        __syncthreads();
        float sterm = 0.f;
        if (tid < TQ * M) {  // the per-job constant || (q - g)_j ||^2, from the raw vectors
            const int q = tid / M, j = tid - q * M;
            if (q < nvq) {
                for (int t = j * dsub; t < (j + 1) * dsub; ++t) {
                    const float df = xs[q * a.dim + t] - gs[t];
                    sterm = fmaf(df, df, sterm);
                }
            }
        }
        __syncthreads();  // (the staged vectors are read; their place is the tables' from here on)
        if (tid < TQ * M) s.sterm[tid] = sterm;
        __syncthreads();
    }
    {
        // the jobs' share and the list's share of every table entry, four entries per thread at
        // a time: their loads first, the sums after
        constexpr int kTurns = (TQ * M * 64 + NW * 64 - 1) / (NW * 64);
        constexpr int kChunk = kTurns < 4 ? kTurns : 4;
        const f32x4 *tab = direct ? nullptr : (const f32x4 *)(a.list_tab + (int64_t)tile_list * (M * 256));
        PSC_LDS f32x4 *dst = (PSC_LDS f32x4 *)s.lut;
#pragma unroll 1
        for (int u0 = 0; u0 < kTurns; u0 += kChunk) {
            f32x4 xv[kChunk], tv[kChunk];
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const int e = tid + (u0 + u) * NW * 64;
                const int q = e / (M * 64), r = e - q * (M * 64);  // r: 16-byte entry of the job's table
                xv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                tv[u] = xv[u];
                if (e < TQ * (M * 64) && q < nvq) {
                    xv[u] = ((const f32x4 *)(a.lut + (direct ? q0 + q : (int64_t)s.gidx[q]) * (M * 256)))[r];
                    if (!direct) tv[u] = tab[r];
                }
            }
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const int e = tid + (u0 + u) * NW * 64;
                const int q = e / (M * 64), r = e - q * (M * 64);
                if (e < TQ * (M * 64)) {
                    f32x4 v = {0.f, 0.f, 0.f, 0.f};
                    if (q < nvq) v = direct ? xv[u] : (xv[u] + tv[u]) + s.sterm[q * M + (r >> 6)];
                    dst[e] = v;
                }
            }
        }
    }
    __syncthreads();
    // arg-min of every table row (lowest index on ties): one wave per row
    for (int row = wave; row < TQ * M; row += NW) {
        const f32x4 v = ((const PSC_LDS f32x4 *)s.lut)[row * 64 + lane];
        float best = v.x;
        int bi = 4 * lane;
        if (v.y < best) { best = v.y; bi = 4 * lane + 1; }
        if (v.z < best) { best = v.z; bi = 4 * lane + 2; }
        if (v.w < best) { best = v.w; bi = 4 * lane + 3; }
        const uint32_t key = dist_key(best);
        const uint32_t wk = wave_min_u32(key);
        const int win = __builtin_ctzll(ballot64(key == wk));  // lower lanes hold lower indices
        const int code = __builtin_amdgcn_readlane(bi, win);
        if (lane == 0) ((PSC_LDS volatile uint8_t *)s.qcw)[row] = (uint8_t)code;
    }
    __syncthreads();
}

// IVF: tiles are (inverted list, up to TQ of its jobs) instead of (query tile, slice).
// SHARE: the workgroups of one query exchange their k-th-best distance through `gthr`; worth
// it when a query is served by many workgroups (inverted lists, four slices or more).
template <int M, int TQ, int NW, bool IVF, bool SHARE>
__global__ void __launch_bounds__(NW * 64)
scan_kernel(ScanArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const Lds<M, TQ> s((PSC_LDS unsigned char *)smem, a.kpad, NW);
    constexpr int WPC = M / 4;       // 32-bit words per code
    constexpr int CB = 32 / TQ;      // codes per lane and block: one survivor bit per (code, query)
    constexpr int NLD = CB * M / 16; // 16-byte loads per lane and block
    constexpr int CPL = 16 / M;      // codes per 16-byte load
    static_assert(CB * TQ == 32 && NLD >= 1, "tile shape");
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // flat mode: tile -> (query tile, database slice); inverted-file mode: tile -> descriptor.
    // [valid_begin, slice_end) is scanned; slice_begin (<= valid_begin) is where positions count
    // from and is a whole number of 16-byte loads into `codes`.
    int slice = 0, tile_list = 0;
    bool whole_db = false;
    int64_t q0, slice_begin, valid_begin, slice_end;
    int nvq;
    if constexpr (IVF) {
        if ((int)blockIdx.x >= *a.ntiles) return;  // the grid is an upper bound on the tile count
        const IvfTile t = a.tiles[blockIdx.x];
        tile_list = t.list;
        q0 = t.job_begin;
        nvq = t.njobs;
        valid_begin = a.list_off[t.list];
        slice_end = a.list_off[t.list + 1];
        slice_begin = valid_begin - valid_begin % CPL;
    } else {
        const FlatTile t = flat_tile(a, blockIdx.x, TQ);
        slice = t.slice;
        whole_db = t.whole;
        q0 = t.q0;
        nvq = (int)((a.nq - q0) < TQ ? (a.nq - q0) : TQ);
        slice_begin = t.slice_begin;
        valid_begin = slice_begin;
        slice_end = t.slice_end;
    }

    const bool spread = a.spread_lists != 0 && nvq == 1;  // (workgroup-uniform)
    // ---- per-slot state
    if (tid < TQ) {
        const int job = spread ? 0 : tid;
        const int gi = job < nvq ? (int)(IVF ? (int64_t)a.job_q[q0 + job] : q0 + job) : -1;
        float t0 = __builtin_inff();
        if constexpr (SHARE) {
            if (gi >= 0 && a.pub_slots == 1)
                t0 = key_dist(__hip_atomic_load(&a.gthr[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
        s.thr[tid] = t0;
        s.lock[tid] = 0;
        s.gidx[tid] = gi;
        s.pslot[tid] = (IVF ? (gi >= 0 ? a.job_slot[q0 + job] : 0) : slice) % a.pub_slots;
    }
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    uint32_t qw[TQ][WPC];  // the tile's query codes, in scalar registers
    if constexpr (IVF) {
        stage_list_tables<M, TQ, NW>(s, a, tile_list, q0, nvq);
        if (tid < nvq * WPC) ((uint32_t *)a.job_qcodes)[q0 * WPC + tid] = s.qcw[tid];
        start_from_published_bounds<M, TQ>(s, a, wave, spread ? TQ : nvq);
        if (spread) {  // every slot gets the job's tables and query code
            PSC_LDS f32x4 *tab = (PSC_LDS f32x4 *)s.lut;
            for (int e = tid; e < (TQ - 1) * (M * 64); e += NW * 64) tab[M * 64 + e] = tab[e % (M * 64)];
            if (tid >= WPC && tid < TQ * WPC) s.qcw[tid] = s.qcw[tid % WPC];
            __syncthreads();
        }
#pragma unroll
        for (int q = 0; q < TQ; ++q) {
#pragma unroll
            for (int w = 0; w < WPC; ++w) qw[q][w] = __builtin_amdgcn_readfirstlane(s.qcw[q * WPC + w]);
        }
    } else {
        // ---- stage the tables
        const f32x4 *src = (const f32x4 *)(a.lut + q0 * (M * 256));
        PSC_LDS f32x4 *dst = (PSC_LDS f32x4 *)s.lut;
        const int nvec = nvq * (M * 256 / 4);
        for (int e = tid; e < TQ * (M * 256 / 4); e += NW * 64) {
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (e < nvec) v = src[e];
            else if (spread) v = src[e % (M * 256 / 4)];  // a single query: every slot gets its tables
            dst[e] = v;
        }
        // ---- query codes -> scalar registers
        const uint32_t *qc = (const uint32_t *)a.qcodes;
#pragma unroll
        for (int q = 0; q < TQ; ++q) {
            const int64_t qq = (q < nvq) ? (q0 + q) : q0;
#pragma unroll
            for (int w = 0; w < WPC; ++w)
                qw[q][w] = __builtin_amdgcn_readfirstlane(qc[qq * WPC + w]);
        }
        __syncthreads();
    }

    // bit TQ-1-q of a code's TQ-bit field <-> query slot q; only the first nvq slots are real
    uint32_t qmask = ((1u << TQ) - 1u) & ~((1u << (TQ - nvq)) - 1u);
    if (spread) qmask = 1u << (TQ - 1 - wave % TQ);  // the wave's own slot
    uint32_t qmask_all = 0u;
#pragma unroll
    for (int c = 0; c < CB; ++c) qmask_all |= qmask << (c * TQ);
    lds_u32 *ring = s.queue + wave * kQueueCap;
    const uint32_t ring_base = (uint32_t)(uintptr_t)ring;  // LDS byte address of the wave's queue
    int fill = 0;  // wave-uniform: entries waiting in the queue (< 64 between turns)
    SharedAsk ask;
    const uint8_t *slice_codes = a.codes + slice_begin * M;
    // graph mode: slot q's own vector sits at position self0 + q of the slice (if it is in there)
    uint32_t self0 = 0x80000000u;
    if (!IVF && a.skip_first >= 0) {
        const int64_t at = a.skip_first + q0 - slice_begin;
        if (at > -64 && at < kMaxSliceLen) self0 = (uint32_t)at;
    }

    const uint32_t bias = a.bias;
    const int64_t stride = (int64_t)NW * 64 * CB;
    const int64_t wave_first = slice_begin + (int64_t)wave * 64 * CB;
    const uint8_t *lane_ptr = a.codes + (wave_first + (int64_t)lane * CB) * M;  // lane's first code

    // The lane's CB consecutive codes as NLD 16-byte loads.  `whole` (wave-uniform) says the
    // wave's block lies entirely inside the slice; otherwise codes past the end read as zero
    // (their survivor bits are masked off below).
    auto load_block = [&](const uint8_t *ptr, int64_t first, bool whole, uint32_t (&w)[CB * WPC]) {
        if (whole) {
#pragma unroll
            for (int l = 0; l < NLD; ++l) {
                const uint4 v = *(const uint4 *)(ptr + l * 16);
                w[l * 4 + 0] = v.x;
                w[l * 4 + 1] = v.y;
                w[l * 4 + 2] = v.z;
                w[l * 4 + 3] = v.w;
            }
        } else {
            const int64_t p = first + (int64_t)lane * CB;
#pragma unroll
            for (int l = 0; l < NLD; ++l) {
                const int64_t pl = p + l * CPL;
                uint32_t *o = &w[l * 4];
                o[0] = o[1] = o[2] = o[3] = 0u;
                if (pl + CPL <= slice_end) {
                    const uint4 v = *(const uint4 *)(ptr + l * 16);
                    o[0] = v.x;
                    o[1] = v.y;
                    o[2] = v.z;
                    o[3] = v.w;
                } else if (CPL == 2 && pl < slice_end) {  // the last, odd 64-bit code
                    const uint2 v = *(const uint2 *)(ptr + l * 16);
                    o[0] = v.x;
                    o[1] = v.y;
                }
            }
        }
    };

    // A wave works on U of its blocks per turn of the main loop ("super-block"): all U filters run
    // back to back (pure VALU) with the U next blocks already asked for, and only then are the U
    // survivor masks queued one after the other -- so a wave waits for memory once per U blocks.
    // (Codes between slice_begin and valid_begin are readable -- they belong to the previous list
    //  -- and are masked off.)
    constexpr int U = (CB * WPC <= 4) ? 4 : (CB * WPC <= 16 ? 2 : 1);
    const int64_t sstride = stride * U;
    uint32_t cur[U][CB * WPC];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t b = wave_first + u * stride;
        if (b < slice_end) load_block(lane_ptr + u * stride * M, b, b + 64 * CB <= slice_end, cur[u]);
    }
    // Lanes without a survivor in a turn write to a private dump word instead of being masked
    // off: cheaper than switching the execution mask twice per turn.
    const uint32_t dump_addr = (uint32_t)(uintptr_t)(s.dump + wave * 64 + lane);
    // One super-block of the wave, starting at code `sb` of the database.  INSIDE: this
    // super-block and the next one lie entirely inside the scanned range, so no code needs masking
    // and the next loads need no bounds -- the form all but the first and last turns take.
    auto superblock = [&](auto inside, const int64_t sb) {
        constexpr bool INSIDE = decltype(inside)::value;
        // ---- Hamming filter: bit c*TQ + (TQ-1-q) of a mask <=> code c is within ht of query q
        uint32_t svs[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t blk = sb + u * stride;
            uint32_t far = 0u;
#pragma unroll
            for (int c = CB - 1; c >= 0; --c) {
                uint32_t wc[WPC];
#pragma unroll
                for (int w = 0; w < WPC; ++w) wc[w] = cur[u][c * WPC + w];
                hamming_test_tile<TQ, WPC>(far, wc, bias, qw);
            }
            uint32_t valid = qmask_all;
            if constexpr (!INSIDE) {
                if (!(blk + 64 * CB <= slice_end && blk >= valid_begin)) {  // ragged or absent block
                    valid = 0u;
#pragma unroll
                    for (int c = 0; c < CB; ++c) {
                        const int64_t p = blk + (int64_t)lane * CB + c;
                        valid |= (p < slice_end && p >= valid_begin) ? (qmask << (c * TQ)) : 0u;
                    }
                }
            }
            svs[u] = ~far & valid;
        }
        // ---- ask for the next super-block
        lane_ptr += sstride * M;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (INSIDE) {
                load_block(lane_ptr + u * stride * M, 0, true, cur[u]);
            } else {
                const int64_t b = sb + sstride + u * stride;
                if (b < slice_end) load_block(lane_ptr + u * stride * M, b, b + 64 * CB <= slice_end, cur[u]);
            }
        }
        // ---- survivors -> queue (one entry per lane and turn), full wavefronts -> ADC
        uint32_t rel0 = (uint32_t)(sb - slice_begin) + (uint32_t)lane * CB;
        auto queue_block = [&](uint32_t sv) {
            while (true) {
                // Queue one survivor bit per lane and turn until no lane has bits left or 64 entries
                // wait.  Hand-scheduled: the compiler's version of this loop spends more scalar
                // instructions on loop control than vector instructions on the work, and every
                // instruction of a wave costs an issue slot.  Per turn: the lanes with a bit are
                // counted (vcc), each takes slot fill + (number of such lanes below it), writes
                // (bit number << kRelBits) | position, and clears that bit; lanes without a bit
                // write to their dump word.  `base` = byte address of queue slot `fill`.
                fill = __builtin_amdgcn_readfirstlane(fill);  // (wave-uniform already; keeps it scalar)
                uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(ring_base + 4u * (uint32_t)fill)), t0, t1, n;
                asm volatile(PSC_QUEUE_TURNS
                             : [sv] "+v"(sv), [fill] "+s"(fill), [base] "+s"(base), [t0] "=&v"(t0), [t1] "=&v"(t1),
                               [n] "=&s"(n)
                             : [rel0] "v"(rel0), [dump] "v"(dump_addr)
                             : "vcc", "scc", "memory");
                static_assert(kRelBits == 27, "the shift in the queueing loop");
                if (fill < 64) break;  // every lane is out of bits
                __builtin_amdgcn_wave_barrier();
                fill -= 64;  // the newest 64 entries go, the others stay where they are
                drain<M, TQ, IVF, SHARE>(s, a, ring + fill, 64, slice_codes, slice_begin, self0, ask);
                __builtin_amdgcn_wave_barrier();
            }
        };
        if constexpr (INSIDE) {  // the hot form: one copy of the queueing code per block, no loop around them
#pragma unroll
            for (int u = 0; u < U; ++u) {
                queue_block(svs[u]);
                rel0 += (uint32_t)stride;
            }
        } else {
#pragma nounroll
            for (int u = 0; u < U; ++u) {
                queue_block(svs[0]);
#pragma unroll
                for (int v = 0; v + 1 < U; ++v) svs[v] = svs[v + 1];  // the next mask moves into place
                rel0 += (uint32_t)stride;
            }
        }
    };
    int64_t sb = wave_first;
    if (sb < slice_end && valid_begin != slice_begin) {  // a list that starts inside a 16-byte load
        superblock(std::false_type{}, sb);
        sb += sstride;
    }
    // turns with two whole super-blocks ahead of sb (computed once, counted in 32 bits)
    const int64_t room = slice_end - sb - (2 * sstride - stride + 64 * CB);
    const int ninside = room >= 0 ? (int)(room / sstride) + 1 : 0;
    for (int i = 0; i < ninside; ++i, sb += sstride) superblock(std::true_type{}, sb);
    for (; sb < slice_end; sb += sstride) superblock(std::false_type{}, sb);
    if (fill > 0) {
        __builtin_amdgcn_wave_barrier();
        drain<M, TQ, IVF, SHARE>(s, a, ring, fill, slice_codes, slice_begin, self0, ask);
    }
    __syncthreads();

    if (spread) {
        // ---- one job, TQ lists: every entry goes to its rank in their union (its place in its
        // own list plus the entries of the other lists below it), the first k ranks are the job's
        int cnt[TQ], total = 0;
#pragma unroll
        for (int t = 0; t < TQ; ++t) {
            cnt[t] = s.lock[t];
            total += cnt[t];
        }
        const int64_t o = IVF ? (int64_t)a.job_slot[q0] * a.k : (q0 * a.nslice + slice) * a.k;
        for (int e = tid; e < TQ * a.k; e += NW * 64) {
            const int t = e / a.k, p = e - t * a.k;
            int mine = 0;
#pragma unroll
            for (int u = 0; u < TQ; ++u) mine = u == t ? cnt[u] : mine;
            if (p >= mine) continue;
            const uint64_t ent = s.top[t * a.kpad + p];
            int rank = p;
#pragma unroll
            for (int u = 0; u < TQ; ++u) {
                if (u == t) continue;
                int lo = 0, hi = cnt[u];  // number of entries of list u below ent
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (s.top[u * a.kpad + mid] < ent) lo = mid + 1; else hi = mid;
                }
                rank += lo;
            }
            if (rank < a.k) {
                a.part_d[o + rank] = entry_dist(ent);
                a.part_i[o + rank] = IVF ? (int64_t)entry_id(ent) : slice_begin + (int64_t)entry_id(ent);
            }
        }
        for (int r = tid; r < a.k; r += NW * 64)
            if (r >= total) {
                a.part_d[o + r] = __builtin_inff();
                a.part_i[o + r] = (int64_t)-1;
            }
        return;
    }
    // ---- write the tile's lists (padded) to the workspace
    for (int e = tid; e < nvq * a.k; e += NW * 64) {
        const int q = e / a.k, r = e - q * a.k;
        const bool have = r < s.lock[q];
        const uint64_t ent = s.top[q * a.kpad + r];
        int64_t o, id;
        if constexpr (IVF) {
            o = (int64_t)a.job_slot[q0 + q] * a.k + r;
            id = (int64_t)entry_id(ent);
        } else {
            o = ((q0 + q) * a.nslice + slice) * a.k + r;
            id = slice_begin + (int64_t)entry_id(ent);
        }
        a.part_d[o] = have ? entry_dist(ent) : __builtin_inff();
        a.part_i[o] = have ? id : (int64_t)-1;
    }
    if constexpr (!IVF) {
        if (whole_db && a.nslice > 1) pad_unused_slices(a, q0, nvq, tid, NW * 64);
    }
}

// ---------------------------------------------------------------------------------------------
// The fused scan with the Hamming test of Section 3.3 ("dual" in Section 4.2) on the matrix cores (64-bit codes, tiles
// of 16 queries, flat and graph mode).  With every bit b written as the byte +1 (b = 0) or -1
// (b = 1), the dot product of two codes is 64 - 2 * (Hamming distance), so
//     distance <= ht   <=>   (2 * ht - 64) + dot >= 0,
// and v_mfma_i32_16x16x64_i8 takes that sum for 16 queries x 16 codes at once when the constant
// goes in as the accumulator: the sign bit of each of the 256 results is the verdict "farther
// than ht".  Per pair that leaves 1/64 of a vector instruction to move the sign into the lane's
// survivor mask, plus the code's share of turning bits into bytes, against five instructions
// of xor / popcount; queue, ADC and lists are those of scan_kernel.
//
// Operand layout (wave64, lane l, col = l % 16, grp = l / 16): the A operand is row `col`
// (query slot col), K positions of group grp; the B operand is column `col` (a code), K
// positions of group grp; lane l receives results (row 4 * grp + r, column col), r = 0..3.
// Both operands give group grp bits 16 * grp .. 16 * grp + 15 of their code, expanded through
// a 256-entry table in LDS (byte -> 8 bytes of +-1): which K positions a group holds does not
// matter as long as both sides agree.
//
// A wave reads 64 codes with one 8-byte load per lane (lane l: code l of the block) and then
// needs, for the four products of the block, the 16-bit part `grp` of codes col, 16 + col,
// 32 + col, 48 + col: a 4 x 4 transpose of 16-bit parts between the four rows of 16 lanes,
// done with one v_permlane32_swap, two v_perm and one v_permlane16_swap.
//
// Survivor masks: bit 31 - (4 * t + r) of a lane's mask <=> (code 16 * t + col of the 128-code
// block, query slot 4 * grp + r), t = 0..7.  Queue entries carry the bit number, grp and the
// position of the block's code `col` (kMfmaRelBits bits).
// ---------------------------------------------------------------------------------------------
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// (One 16-wave workgroup per compute unit = 4 waves per SIMD: telling the compiler so lets it
//  spend registers on keeping the eight products of a block in flight together.)
// IVF: tiles are (inverted list, up to 16 of its jobs), as in scan_kernel.
template <int NW, bool SHARE, bool IVF = false>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
scan_mfma_kernel(ScanArgs a)
{
    constexpr int M = 8, TQ = 16;
    constexpr int kBlock = 128;  // codes per wave and turn
    extern __shared__ __align__(16) unsigned char smem[];
    // [256] byte -> eight bytes of +-1, at LDS address 0 so that a look-up address is just byte * 8
    PSC_LDS u32x2 *xtab = (PSC_LDS u32x2 *)smem;
    const Lds<M, TQ> s((PSC_LDS unsigned char *)smem + kMfmaTableBytes, a.kpad, NW);
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, grp = lane >> 4;

    FlatTile ft{};
    int slice = 0, tile_list = 0;
    int64_t q0, slice_begin, slice_end;
    int nvq;
    if constexpr (IVF) {
        if ((int)blockIdx.x >= *a.ntiles) return;  // the grid is an upper bound on the tile count
        const IvfTile t = a.tiles[blockIdx.x];
        tile_list = t.list;
        q0 = t.job_begin;
        nvq = t.njobs;
        slice_begin = a.list_off[t.list];  // (8-byte loads, one code each: a list may start anywhere)
        slice_end = a.list_off[t.list + 1];
    } else {
        ft = flat_tile(a, blockIdx.x, TQ);
        slice = ft.slice;
        q0 = ft.q0;
        nvq = (int)((a.nq - q0) < TQ ? (a.nq - q0) : TQ);
        slice_begin = ft.slice_begin;
        slice_end = ft.slice_end;
    }
    // the look-ups below take the table to start at LDS address 0, the queue entries a position
    // in kMfmaRelBits bits: flag the run instead of returning something wrong
    if ((uint32_t)(uintptr_t)xtab != 0u || slice_end - slice_begin > kMfmaMaxSliceLen) {
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }

    if (tid < TQ) {
        const int gi = tid < nvq ? (int)(IVF ? (int64_t)a.job_q[q0 + tid] : q0 + tid) : -1;
        float t0 = __builtin_inff();
        if constexpr (SHARE) {
            if (gi >= 0 && a.pub_slots == 1)
                t0 = key_dist(__hip_atomic_load(&a.gthr[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
        s.thr[tid] = t0;
        s.lock[tid] = 0;
        s.gidx[tid] = gi;
        s.pslot[tid] = (IVF ? (gi >= 0 ? a.job_slot[q0 + tid] : 0) : slice) % a.pub_slots;
    }
    for (int v = tid; v < 256; v += NW * 64) {
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i >> 2] |= (((v >> i) & 1) ? 0xffu : 0x01u) << (8 * (i & 3));
        xtab[v] = u32x2{w[0], w[1]};
    }
    if constexpr (IVF) {
        stage_list_tables<M, TQ, NW>(s, a, tile_list, q0, nvq);
        if (tid < nvq * 2) ((uint32_t *)a.job_qcodes)[q0 * 2 + tid] = s.qcw[tid];
        start_from_published_bounds<M, TQ>(s, a, wave, nvq);
    } else {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 *src = (const f32x4 *)(a.lut + q0 * (M * 256));
        PSC_LDS f32x4 *dst = (PSC_LDS f32x4 *)s.lut;
        const int nvec = nvq * (M * 256 / 4);
        for (int e = tid; e < TQ * (M * 256 / 4); e += NW * 64) {
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (e < nvec) v = src[e];
            dst[e] = v;
        }
        __syncthreads();
    }

    // A operand: part grp of query slot col (slots past nvq: any code, their results are masked)
    i32x4 qa;
    {
        uint32_t q16;
        if constexpr (IVF)
            q16 = ((const PSC_LDS uint16_t *)s.qcw)[(col < nvq ? col : 0) * 4 + grp];
        else
            q16 = ((const uint16_t *)a.qcodes)[(q0 + (col < nvq ? col : 0)) * 4 + grp];
        const u32x2 lo = xtab[q16 & 0xffu], hi = xtab[q16 >> 8];
        qa = i32x4{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
    }
    const int ht = (int)(0x7fffffffu - a.bias);
    const int c0 = 2 * ht - 64;
    const i32x4 cinit = {c0, c0, c0, c0};
    uint32_t valid_q = 0u;  // the lane's rows that are real queries, for all eight groups of codes
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (4 * grp + r < nvq) valid_q |= 0x11111111u << (3 - r);

    lds_u32 *ring = s.queue + wave * kQueueCap;
    const uint32_t ring_base = (uint32_t)(uintptr_t)ring;
    const uint32_t dump_addr = (uint32_t)(uintptr_t)(s.dump + wave * 64 + lane);
    int fill = 0;
    SharedAsk ask;
    const uint8_t *slice_codes = a.codes + slice_begin * M;
    uint32_t self0 = 0x80000000u;
    if (!IVF && a.skip_first >= 0) {
        const int64_t at = a.skip_first + q0 - slice_begin;
        if (at > -64 && at < kMfmaMaxSliceLen) self0 = (uint32_t)at;
    }
    const uint32_t lane_bits = (uint32_t)col | ((uint32_t)grp << kMfmaRelBits);

    auto queue_block = [&](uint32_t sv, const uint32_t rel0) {
        while (true) {
            fill = __builtin_amdgcn_readfirstlane(fill);
            uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(ring_base + 4u * (uint32_t)fill)), t0, t1, n;
            asm volatile(PSC_QUEUE_TURNS
                         : [sv] "+v"(sv), [fill] "+s"(fill), [base] "+s"(base), [t0] "=&v"(t0), [t1] "=&v"(t1),
                           [n] "=&s"(n)
                         : [rel0] "v"(rel0), [dump] "v"(dump_addr)
                         : "vcc", "scc", "memory");
            if (fill < 64) break;
            __builtin_amdgcn_wave_barrier();
            fill -= 64;
            drain<M, TQ, IVF, SHARE, true>(s, a, ring + fill, 64, slice_codes, slice_begin, self0, ask);
            __builtin_amdgcn_wave_barrier();
        }
    };

    // The wave's blocks: wave, wave + NW, ... of the slice's 128-code blocks; the next block's
    // codes are asked for before the current one is worked on.  WHOLE: the block lies entirely
    // inside the slice (all but the last turn or two of a wave).
    const int64_t stride = (int64_t)NW * kBlock;
    auto load_block = [&](auto whole, int64_t blk, uint2 (&c)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t p = blk + 64 * h + lane;
            if constexpr (decltype(whole)::value) {
                c[h] = *(const uint2 *)(a.codes + p * M);
            } else {
                c[h] = make_uint2(0u, 0u);
                if (p < slice_end) c[h] = *(const uint2 *)(a.codes + p * M);
            }
        }
    };
    auto filter_block = [&](auto whole, int64_t blk, const uint2 (&c)[2]) {
        // In three phases kept apart for the scheduler (left alone it runs the eight products one
        // after the other, each waiting for its table entries and then for its own result):
        // all sixteen look-ups, the eight products, the thirty-two sign bits.
        i32x4 cb[8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // rows 0,1 get the low words of all four rows' codes, rows 2,3 the high words ...
            const auto r32 = __builtin_amdgcn_permlane32_swap(c[h].x, c[h].y, false, false);
            // ... sorted by 16-bit part ...
            uint32_t pa = __builtin_amdgcn_perm(r32[1], r32[0], 0x05040100u);
            uint32_t pb = __builtin_amdgcn_perm(r32[1], r32[0], 0x07060302u);
            // ... and odd rows trade their even parts for the even rows' odd parts: row grp now
            // holds part grp of the codes of rows 0 (pa low), 1 (pb low), 2 (pa high), 3 (pb high)
            const auto r16 = __builtin_amdgcn_permlane16_swap(pa, pb, false, false);
            pa = r16[0];
            pb = r16[1];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t src = (t & 1) ? pb : pa;
                const uint32_t c16 = (t & 2) ? (src >> 16) : (src & 0xffffu);
                // (the table starts at LDS address 0: a look-up address is the byte times 8, which
                //  the compiler then takes straight out of the word with a byte-select shift)
                const u32x2 lo = *(PSC_LDS u32x2 *)(uintptr_t)((c16 & 0xffu) << 3);
                const u32x2 hi = *(PSC_LDS u32x2 *)(uintptr_t)((c16 >> 8) << 3);
                cb[4 * h + t] = i32x4{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        i32x4 acc[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa, cb[t], cinit, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        uint32_t far = 0u;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
#pragma unroll
            for (int r = 0; r < 4; ++r) far = __builtin_amdgcn_alignbit(far, (uint32_t)acc[t][r], 31);
        }
        uint32_t valid = valid_q;
        if constexpr (!decltype(whole)::value) {  // ragged block: codes past the end do not count
            uint32_t in = 0u;
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (blk + 16 * t + col < slice_end) in |= 0xf0000000u >> (4 * t);
            valid &= in;
        }
        queue_block(~far & valid, (uint32_t)(blk - slice_begin) + lane_bits);
    };
    uint2 cur[2];
    int64_t blk = slice_begin + (int64_t)wave * kBlock;
    if (blk < slice_end) load_block(std::false_type{}, blk, cur);
    while (blk + stride + kBlock <= slice_end) {  // this block and the next are whole
        uint2 nxt[2];
        load_block(std::true_type{}, blk + stride, nxt);
        filter_block(std::true_type{}, blk, cur);
        cur[0] = nxt[0];
        cur[1] = nxt[1];
        blk += stride;
    }
    for (; blk < slice_end; blk += stride) {
        uint2 nxt[2] = {make_uint2(0u, 0u), make_uint2(0u, 0u)};
        if (blk + stride < slice_end) load_block(std::false_type{}, blk + stride, nxt);
        filter_block(std::false_type{}, blk, cur);
        cur[0] = nxt[0];
        cur[1] = nxt[1];
    }
    if (fill > 0) {
        __builtin_amdgcn_wave_barrier();
        drain<M, TQ, IVF, SHARE, true>(s, a, ring, fill, slice_codes, slice_begin, self0, ask);
    }
    __syncthreads();

    for (int e = tid; e < nvq * a.k; e += NW * 64) {
        const int q = e / a.k, r = e - q * a.k;
        const bool have = r < s.lock[q];
        const uint64_t ent = s.top[q * a.kpad + r];
        int64_t o, id;
        if constexpr (IVF) {
            o = (int64_t)a.job_slot[q0 + q] * a.k + r;
            id = (int64_t)entry_id(ent);
        } else {
            o = ((q0 + q) * a.nslice + slice) * a.k + r;
            id = slice_begin + (int64_t)entry_id(ent);
        }
        a.part_d[o] = have ? entry_dist(ent) : __builtin_inff();
        a.part_i[o] = have ? id : (int64_t)-1;
    }
    if constexpr (!IVF) {
        if (ft.whole && a.nslice > 1) pad_unused_slices(a, q0, nvq, tid, NW * 64);
    }
}

// ---------------------------------------------------------------------------------------------
// Pure ADC scan: ht >= 8m keeps every code (Section 4.2 "ADC", the PQ baseline of the paper), so
// there is nothing to filter or to queue: every (query, code) pair is scored.  The bound is the
// LDS gather rate, so the TQ tables are interleaved in LDS four queries to an entry,
// lut4[g][j][c] = (T_{4g}[j][c], .., T_{4g+3}[j][c]): one 16-byte read serves four queries of
// the tile, and a code's m byte offsets are computed once for all TQ queries.
// Same tiling (query tile x database slice), lists, ordering and outputs as scan_kernel.
// FILTER: the Hamming test of Section 3.3 is still applied -- to the pairs whose distance beats the
// current k-th best, which are few; since that k-th best is taken among pairs that pass the test,
// the outcome is the one of testing every pair first.  This is the cheaper route when the
// threshold lets a large share of the codes through: scoring everything from the interleaved
// tables then costs less than queueing the survivors one by one.
// ---------------------------------------------------------------------------------------------
template <int M, int TQ, int NW, bool SHARE, bool FILTER>
__global__ void __launch_bounds__(NW * 64)
adc_kernel(ScanArgs a)
{
    static_assert(TQ % 4 == 0, "four queries per table entry");
    extern __shared__ __align__(16) unsigned char smem[];
    const Lds<M, TQ> s((PSC_LDS unsigned char *)smem, a.kpad, NW);
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int G = TQ / 4;
    constexpr int WPC = M / 4;
    constexpr int CPL = 16 / M;  // codes per 16-byte load
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const FlatTile ft = flat_tile(a, blockIdx.x, TQ);
    const int slice = ft.slice;
    const int64_t q0 = ft.q0;
    const int nvq = (int)((a.nq - q0) < TQ ? (a.nq - q0) : TQ);
    const int64_t slice_begin = ft.slice_begin;
    const int64_t slice_end = ft.slice_end;

    // ---- stage the tables interleaved, reset the lists
    {
        const float *src = a.lut + q0 * (M * 256);
        PSC_LDS float *dst = (PSC_LDS float *)s.lut;
        for (int e = tid; e < TQ * M * 256; e += NW * 64) {
            const int q = e / (M * 256), r = e - q * (M * 256);
            dst[(((q >> 2) * (M * 256) + r) << 2) + (q & 3)] = q < nvq ? src[e] : 0.f;
        }
        if (tid < TQ) {
            float t0 = __builtin_inff();
            if constexpr (SHARE) {
                if (tid < nvq && a.pub_slots == 1)
                    t0 = key_dist(__hip_atomic_load(&a.gthr[q0 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            }
            s.thr[tid] = t0;
            s.lock[tid] = 0;
            s.gidx[tid] = tid < nvq ? (int)(q0 + tid) : -1;
            s.pslot[tid] = slice % a.pub_slots;
        }
    }
    // ---- query codes -> scalar registers (only the filtering variant reads them)
    uint32_t qw[TQ][WPC];
    if constexpr (FILTER) {
        const uint32_t *qc = (const uint32_t *)a.qcodes;
#pragma unroll
        for (int q = 0; q < TQ; ++q) {
            const int64_t qq = (q < nvq) ? (q0 + q) : q0;
#pragma unroll
            for (int w = 0; w < WPC; ++w) qw[q][w] = __builtin_amdgcn_readfirstlane(qc[qq * WPC + w]);
        }
    }
    __syncthreads();

    const PSC_LDS f32x4 *lut4 = (const PSC_LDS f32x4 *)s.lut;
    SharedAsk ask;
    const int64_t stride = (int64_t)NW * 64 * CPL;
    const int64_t skip_rel = a.skip_first + q0 - slice_begin;
    const bool skipping = a.skip_first >= 0 && skip_rel > -(int64_t)TQ && skip_rel < kMaxSliceLen;
    for (int64_t blk = slice_begin + (int64_t)wave * 64 * CPL; blk < slice_end; blk += stride) {
        const int64_t p0 = blk + (int64_t)lane * CPL;
        uint32_t shared = kKeyInf;
        const bool asking = SHARE && ask.wanted;
        if (asking) shared = ask_shared_thresholds<M, TQ>(s, a);
        ask.wanted = false;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (p0 + CPL <= slice_end) {
            const uint4 v = *(const uint4 *)(a.codes + p0 * M);
            w[0] = v.x;
            w[1] = v.y;
            w[2] = v.z;
            w[3] = v.w;
        } else if (CPL == 2 && p0 < slice_end) {
            const uint2 v = *(const uint2 *)(a.codes + p0 * M);
            w[0] = v.x;
            w[1] = v.y;
        }
        if (asking) adopt_shared_thresholds<M, TQ>(s, shared);
        // thresholds of the tile, refreshed once per block: lane q holds thr[q]
        const float thr_v = s.thr[lane & (TQ - 1)];
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const bool live = p0 + c < slice_end;
            const uint32_t rel = (uint32_t)(p0 + c - slice_begin);
            uint32_t off[M];  // the code's byte for sub-quantizer j = its entry in sub-table j
#pragma unroll
            for (int j = 0; j < M; ++j) off[j] = ((w[c * WPC + (j >> 2)] >> (8 * (j & 3))) & 0xffu);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                f32x4 acc = lut4[(g * M + 0) * 256 + off[0]];
#pragma unroll
                for (int j = 1; j < M; ++j) acc += lut4[(g * M + j) * 256 + off[j]];
                float d[4] = {acc.x, acc.y, acc.z, acc.w};
                uint64_t any = 0;
                bool pass[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int q = g * 4 + i;
                    const float thr = bcast_f(thr_v, q);
                    pass[i] = live && q < nvq && d[i] <= thr;
                    if (skipping) pass[i] = pass[i] && rel != (uint32_t)((int32_t)skip_rel + q);
                    any |= ballot64(pass[i]);
                }
                if (any) {
                    // FILTER: the Hamming test is taken only here, on the few pairs whose distance
                    // beats the threshold (which is the k-th best among the pairs that pass the test:
                    // the result is that of testing every pair), not on every pair of the stream.
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if constexpr (FILTER) {  // bias + h overflows into the sign bit iff h > ht
                            const int q = g * 4 + i;
                            uint32_t acc = a.bias;
#pragma unroll
                            for (int ww = 0; ww < WPC; ++ww) acc += (uint32_t)__popc(w[c * WPC + ww] ^ qw[q][ww]);
                            pass[i] = pass[i] && (int32_t)acc >= 0;
                        }
                        const uint64_t mine = ballot64(pass[i]);
                        if (mine) {
                            ask.wanted = true;
                            insert_candidates<M, TQ, SHARE, SHARE>(s, a, g * 4 + i, mine, d[i], rel);
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    for (int e = tid; e < nvq * a.k; e += NW * 64) {
        const int q = e / a.k, r = e - q * a.k;
        const bool have = r < s.lock[q];
        const uint64_t ent = s.top[q * a.kpad + r];
        const int64_t o = ((q0 + q) * a.nslice + slice) * a.k + r;
        a.part_d[o] = have ? entry_dist(ent) : __builtin_inff();
        a.part_i[o] = have ? (slice_begin + (int64_t)entry_id(ent)) : (int64_t)-1;
    }
    if (ft.whole && a.nslice > 1) pad_unused_slices(a, q0, nvq, tid, NW * 64);
}

// Merge the nslice sorted partial lists of each query into the final k (one wave per query).
// Lane l owns lists l, l + 64, ...: it keeps the head of each in registers together with the
// entry after it, so that a step of the merge (pick the smallest head of the wave, advance that
// list) waits for memory only when one list wins several times in a row.  Padding entries
// (id < 0) end a list.
template <int OWN>
__global__ void __launch_bounds__(64)
merge_kernel(const float *__restrict__ part_d, const int64_t *__restrict__ part_i, int nslice, int k,
             int64_t id_base, const int *__restrict__ status, int64_t *__restrict__ ids,
             float *__restrict__ dists)
{
    const int64_t q = blockIdx.x;
    const int lane = lane_id();
    const float *pd = part_d + q * nslice * k;
    const int64_t *pi = part_i + q * nslice * k;
    const bool poisoned = *status != 0;
    uint32_t hk[OWN], nk[OWN];  // distance keys of the head and of the entry after it (kKeyNone: none)
    int64_t hi[OWN], ni[OWN];   // their ids
    int pos[OWN];               // index of the head in its list
    constexpr uint32_t kKeyNone = 0xffffffffu;  // above every real key, +infinity included
    auto fetch = [&](int l, int at, uint32_t &key, int64_t &id) {
        key = kKeyNone;
        id = -1;
        if (l < nslice && at < k) {
            const int64_t i = pi[(int64_t)l * k + at];
            if (i >= 0) {
                id = i;
                key = dist_key(pd[(int64_t)l * k + at]);
            }
        }
    };
#pragma unroll
    for (int t = 0; t < OWN; ++t) {
        pos[t] = 0;
        fetch(lane + 64 * t, 0, hk[t], hi[t]);
        fetch(lane + 64 * t, 1, nk[t], ni[t]);
    }
    for (int r = 0; r < k; ++r) {
        // the lane's best head
        uint32_t bk = hk[0];
        int64_t bi = hi[0];
        int bt = 0;
#pragma unroll
        for (int t = 1; t < OWN; ++t) {
            if (hk[t] < bk || (hk[t] == bk && hk[t] != kKeyNone && hi[t] < bi)) {
                bk = hk[t];
                bi = hi[t];
                bt = t;
            }
        }
        // the wave's: smallest key, and the lowest id among the lanes that hold it
        const uint32_t wk = wave_min_u32(bk);
        uint64_t tied = ballot64(bk == wk);
        int win = __builtin_ctzll(tied);
        if (wk != kKeyNone && (tied & (tied - 1))) {
            int64_t best = INT64_MAX;
            while (tied) {
                const int l = __builtin_ctzll(tied);
                tied &= tied - 1;
                const int64_t cand = ((int64_t)__builtin_amdgcn_readlane((int)(bi >> 32), l) << 32) |
                                     (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bi, l);
                if (cand < best) {
                    best = cand;
                    win = l;
                }
            }
        }
        const bool have = wk != kKeyNone;
        const int64_t wi = ((int64_t)__builtin_amdgcn_readlane((int)(bi >> 32), win) << 32) |
                           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bi, win);
        if (lane == 0) {
            ids[q * k + r] = poisoned ? (int64_t)-2 : (have ? wi + id_base : (int64_t)-1);
            dists[q * k + r] = have ? key_dist(wk) : __builtin_inff();
        }
        if (have && lane == win) {  // advance the winning list
#pragma unroll
            for (int t = 0; t < OWN; ++t) {
                if (t == bt) {
                    hk[t] = nk[t];
                    hi[t] = ni[t];
                    ++pos[t];
                    fetch(lane + 64 * t, pos[t] + 1, nk[t], ni[t]);
                }
            }
        }
    }
}

// The same merge for a handful of queries, where the hundred dependent steps of the wave above are
// all there is to wait for: a workgroup of 16 waves per query selects the k smallest
// (distance, id) pairs of all partial lists at once.  Thread t holds the distance keys of
// entries t, t + 1024, ... of the query's lists; the k-th smallest key is found bit by bit with
// one workgroup-wide count per bit (per-wave sums through LDS, two buffers in turn so that one
// barrier per bit is enough); if more entries than needed share it, the same search over the bits
// of the id finds the last id that belongs.  The selected entries go to LDS in any order and each
// is written to its rank.
constexpr int64_t kMergeSelectQueries = 32;      // up to this many queries,
constexpr int64_t kMergeSelectManyQueries = 512; // or this many if each has 32 lists or more (probed lists:
                                                 // 10k queries x 64 probes of 100M vectors, whole search, with the
                                                 // wave above / with this kernel: 64 queries 0.45 / 0.34 ms,
                                                 // 256: 0.61 / 0.57, 512: 0.84 / 0.81, 1024: 1.31 / 1.32)
constexpr int64_t kMergeSelectEntries = 32768;   // and this many entries per query
// (its forty-odd counting steps take about 20 us whatever k is; the wave above takes 0.4 us per
//  result: measured 32 against 42 us at k = 100, 20 against 5 us at k = 10)
constexpr int kMergeSelectMinK = 64;

// Sum of v over the wave, in every lane (row-local steps on the data-parallel path, the four row
// sums through scalar registers).
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);   // lane ^ 1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);   // lane ^ 2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);  // mirror in 8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, false);  // mirror in 16
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

template <int KPL>
__global__ void __launch_bounds__(1024)
merge_select_kernel(const float *__restrict__ part_d, const int64_t *__restrict__ part_i, int nslice, int k,
                    const int *__restrict__ status, int64_t *__restrict__ ids, float *__restrict__ dists)
{
    __shared__ uint32_t part[2][16];
    __shared__ __align__(16) uint32_t selk[1024];
    __shared__ int64_t seli[1024];
    __shared__ uint32_t nsel;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t q = blockIdx.x;
    // Rank of (key, id) among the n selected entries in LDS: keys are compared four to a read; the
    // ids are looked at only by a thread whose key occurs more than once.
    auto rank_among = [&](uint32_t key, int64_t id, int n) {
        int lt = 0, eq = 0;
        const int n4 = n & ~3;
        for (int j = 0; j < n4; j += 4) {
            const uint4 v = *(const uint4 *)&selk[j];
            lt += (v.x < key ? 1 : 0) + (v.y < key ? 1 : 0) + (v.z < key ? 1 : 0) + (v.w < key ? 1 : 0);
            eq += (v.x == key ? 1 : 0) + (v.y == key ? 1 : 0) + (v.z == key ? 1 : 0) + (v.w == key ? 1 : 0);
        }
        for (int j = n4; j < n; ++j) {
            lt += selk[j] < key ? 1 : 0;
            eq += selk[j] == key ? 1 : 0;
        }
        if (eq > 1)
            for (int j = 0; j < n; ++j) lt += (selk[j] == key && seli[j] < id) ? 1 : 0;
        return lt;
    };
    const int total = nslice * k;
    const float *pd = part_d + q * total;
    const int64_t *pi = part_i + q * total;
    const bool poisoned = *status != 0;
    constexpr uint32_t kNone = 0xffffffffu;  // padding and places past the end; real keys stay below
    // (Places a list does not fill hold distance +infinity, which no scored code has: the distances
    //  alone tell them apart, so all loads of a thread are independent of one another and in flight
    //  together -- one trip to memory instead of one per entry.)
    uint32_t dk[KPL];
    {
        float dv[KPL];
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            const int e = i * 1024 + tid;
            dv[i] = pd[e < total ? e : total - 1];
        }
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            const int e = i * 1024 + tid;
            dk[i] = (e < total && dv[i] != __builtin_inff()) ? min(dist_key(dv[i]), kNone - 1u) : kNone;
        }
    }
    if (tid == 0) nsel = 0u;
    int turn = 0;
    // number of the workgroup's entries for which pred(i) holds (a second predicate is counted in
    // the high half of the word)
    auto count = [&](auto pred, auto... more) {
        uint32_t cnt = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            cnt += pred(i) ? 1u : 0u;
            ((cnt += more(i) ? 0x10000u : 0u), ...);
        }
        cnt = wave_sum_u32(cnt);
        if (lane == 0) part[turn][wave] = cnt;
        __syncthreads();
        uint32_t all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) all += part[turn][w];
        turn ^= 1;
        return all;
    };
    // A bound on the k-th smallest key from single rows of the (sorted) lists: if t lists have their
    // r-th entry at or below v, at least t (r + 1) entries lie at or below v, so for any t <= nslice
    // the t-th smallest key of row ceil(k / t) - 1 bounds the k-th smallest of all.  Lists of equal
    // quality (the slices of a flat scan) make the widest t the sharpest -- with 256 lists the 100th
    // smallest head --, lists of unequal quality (the probed lists of an inverted file: the
    // nearest few hold nearly all of the answer) a small t on a deep row; wave w tries t = T >> w, T
    // the widest, down to t = 1, and the smallest of their values is taken.  That usually leaves a
    // few hundred entries of tens of thousands, which are ranked directly instead of being searched
    // bit by bit (three barriers instead of forty).
    __shared__ uint32_t bounds_s[16];
    {
        const int row0 = (k + nslice - 1) / nslice - 1;
        const uint32_t t_widest = (uint32_t)((k + row0) / (row0 + 1));  // (<= nslice)
        const uint32_t t = max(t_widest >> wave, 1u);
        const bool active = wave == 0 || (t_widest >> (wave - 1)) > 1u;  // (t = 1 is tried once)
        uint32_t b0 = kNone;
        if (active) {
            const int row = (k + (int)t - 1) / (int)t - 1;  // t (row + 1) >= k, row <= k - 1
            uint32_t rk[16];  // the row, 16 keys to a lane (nslice <= 1024)
            const int nreg = (nslice + 63) >> 6;  // (wave-uniform)
            {
                float rv[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int l = i * 64 + lane;
                    rv[i] = (i < nreg && l < nslice) ? pd[(int64_t)l * k + row] : __builtin_inff();
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) rk[i] = rv[i] != __builtin_inff() ? min(dist_key(rv[i]), kNone - 1u) : kNone;
            }
            b0 = 0;  // the t-th smallest key of the row (kNone when the row has fewer than t entries)
            for (int b = 31; b >= 0; --b) {
                const uint32_t mid = b0 | (1u << b);
                uint32_t cnt = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (i < nreg) cnt += rk[i] < mid ? 1u : 0u;
                if (wave_sum_u32(cnt) < t) b0 = mid;
            }
        }
        if (lane == 0) bounds_s[wave] = b0;
    }
    __syncthreads();
    uint32_t bound = bounds_s[0];
#pragma unroll
    for (int w = 1; w < 16; ++w) bound = min(bound, bounds_s[w]);
    // entries that exist (low half) and entries at or below the bound (high half), in one count
    // (at most 32768 entries: each half fits 16 bits)
    const uint32_t both = count([&](int i) { return dk[i] != kNone; }, [&](int i) { return bound != kNone && dk[i] <= bound; });
    const uint32_t have = both & 0xffffu;
    const uint32_t kk = have < (uint32_t)k ? have : (uint32_t)k;  // entries to return
    const uint32_t near = bound == kNone ? 1025u : both >> 16;
    if (kk > 0 && near <= 1024u) {
        // (near >= kk: the bound is at or above the k-th smallest key)
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            if (dk[i] > bound) continue;
            const uint32_t slot = atomicAdd(&nsel, 1u);
            selk[slot] = dk[i];
            seli[slot] = pi[i * 1024 + tid];
        }
        __syncthreads();
        if (tid < (int)near) {
            const uint32_t key = selk[tid];
            const int64_t id = seli[tid];
            const int rank = rank_among(key, id, (int)near);
            if (rank < (int)kk) {
                ids[q * k + rank] = poisoned ? (int64_t)-2 : id;
                dists[q * k + rank] = key_dist(key);
            }
        }
        if (tid >= (int)kk && tid < k) {
            ids[q * k + tid] = poisoned ? (int64_t)-2 : (int64_t)-1;
            dists[q * k + tid] = __builtin_inff();
        }
        return;
    }
    if (kk > 0) {
        uint32_t pivot = 0;  // the kk-th smallest key
        for (int b = 31; b >= 0; --b) {
            const uint32_t mid = pivot | (1u << b);
            if (count([&](int i) { return dk[i] < mid; }) < kk) pivot = mid;
        }
        const uint32_t below = count([&](int i) { return dk[i] < pivot; });
        const uint32_t upto = count([&](int i) { return dk[i] <= pivot; });
        int64_t last = INT64_MAX;  // entries at the pivot distance belong up to this id
        if (upto > kk) {
            int64_t eid[KPL];
#pragma unroll
            for (int i = 0; i < KPL; ++i) eid[i] = dk[i] == pivot ? pi[i * 1024 + tid] : INT64_MAX;
            const uint32_t want = kk - below;  // >= 1
            int64_t lp = 0;
            for (int b = 62; b >= 0; --b) {
                const int64_t mid = lp | ((int64_t)1 << b);
                if (count([&](int i) { return eid[i] < mid; }) < want) lp = mid;
            }
            last = lp;
        }
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            if (dk[i] > pivot) continue;
            const int64_t id = pi[i * 1024 + tid];
            if (dk[i] == pivot && id > last) continue;
            const uint32_t slot = atomicAdd(&nsel, 1u);
            if (slot < 1024u) {  // (exactly kk <= 1024 entries pass)
                selk[slot] = dist_key(pd[i * 1024 + tid]);
                seli[slot] = id;
            }
        }
    }
    __syncthreads();
    if (tid < (int)kk) {
        const uint32_t key = selk[tid];
        const int64_t id = seli[tid];
        const int rank = rank_among(key, id, (int)kk);
        ids[q * k + rank] = poisoned ? (int64_t)-2 : id;
        dists[q * k + rank] = key_dist(key);
    } else if (tid < k) {
        ids[q * k + tid] = poisoned ? (int64_t)-2 : (int64_t)-1;
        dists[q * k + tid] = __builtin_inff();
    }
}

// One wave per query; the lists are spread over the lanes, OWN to a lane.
int launch_merge(const float *part_d, const int64_t *part_i, int64_t nq, int nlists, int k, const int *status,
                 int64_t *ids, float *dists, hipStream_t s)
{
    PSC_REQUIRE(nlists >= 1 && nlists <= 1024, "between 1 and 1024 partial lists per query, got %d", nlists);
    const dim3 grid((unsigned)nq), block(64);
    if ((nq <= kMergeSelectQueries || (nq <= kMergeSelectManyQueries && nlists >= 32)) &&
        (int64_t)nlists * k <= kMergeSelectEntries && k >= kMergeSelectMinK && k <= 1024) {
        if ((int64_t)nlists * k <= 8 * 1024)
            hipLaunchKernelGGL(merge_select_kernel<8>, grid, dim3(1024), 0, s, part_d, part_i, nlists, k, status, ids, dists);
        else
            hipLaunchKernelGGL(merge_select_kernel<32>, grid, dim3(1024), 0, s, part_d, part_i, nlists, k, status, ids, dists);
        PSC_HIP_TRY(hipGetLastError());
        return PSC_OK;
    }
    if (nlists <= 64)
        hipLaunchKernelGGL(merge_kernel<1>, grid, block, 0, s, part_d, part_i, nlists, k, (int64_t)0, status, ids, dists);
    else if (nlists <= 128)
        hipLaunchKernelGGL(merge_kernel<2>, grid, block, 0, s, part_d, part_i, nlists, k, (int64_t)0, status, ids, dists);
    else if (nlists <= 256)
        hipLaunchKernelGGL(merge_kernel<4>, grid, block, 0, s, part_d, part_i, nlists, k, (int64_t)0, status, ids, dists);
    else
        hipLaunchKernelGGL(merge_kernel<16>, grid, block, 0, s, part_d, part_i, nlists, k, (int64_t)0, status, ids, dists);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

__global__ void fill_padding_kernel(int64_t *ids, float *dists, int64_t total)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) {
        ids[e] = -1;
        dists[e] = __builtin_inff();
    }
}

// Start of a scan: every shared threshold at +infinity and, if asked, the status word cleared.
__global__ void init_scan_kernel(uint32_t *gthr, int64_t n, int *status)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) gthr[e] = kKeyInf;
    if (e == 0 && status) *status = 0;
}

// Hamming filter alone: per query the number of codes within ht (and optionally every distance).
// A workgroup column serves kFilterTQ queries at a time, so that a code is loaded once for all of
// them (their code words are the same for every lane: scalar registers).
constexpr int kFilterTQ = 16;
template <int M>
__global__ void __launch_bounds__(256)
hamming_filter_kernel(const uint8_t *__restrict__ qcodes, int64_t nq, const uint8_t *__restrict__ codes,
                      int64_t n, int ht, unsigned long long *__restrict__ nsurv,
                      uint8_t *__restrict__ hdist)
{
    constexpr int WPC = M / 4;
    const int64_t q0 = (int64_t)blockIdx.y * kFilterTQ;
    const int nvq = (int)((nq - q0) < kFilterTQ ? (nq - q0) : kFilterTQ);
    uint32_t qw[kFilterTQ][WPC];
#pragma unroll
    for (int t = 0; t < kFilterTQ; ++t) {
        const int64_t q = q0 + (t < nvq ? t : 0);
#pragma unroll
        for (int w = 0; w < WPC; ++w) qw[t][w] = ((const uint32_t *)qcodes)[q * WPC + w];
    }
    uint32_t local[kFilterTQ];
#pragma unroll
    for (int t = 0; t < kFilterTQ; ++t) local[t] = 0u;
    // (a thread counts at most n / (256 * gridDim.x) < 2^32 codes per query)
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        uint32_t cw[WPC];
#pragma unroll
        for (int w = 0; w < WPC; ++w) cw[w] = ((const uint32_t *)codes)[i * WPC + w];
#pragma unroll
        for (int t = 0; t < kFilterTQ; ++t) {
            int h = 0;
#pragma unroll
            for (int w = 0; w < WPC; ++w) h += __popc(cw[w] ^ qw[t][w]);
            if (hdist && t < nvq) hdist[(q0 + t) * n + i] = (uint8_t)h;
            local[t] += (h <= ht) ? 1u : 0u;
        }
    }
    // wave reduction, workgroup reduction, then one atomic per workgroup and query (many waves
    // adding to the same few counters would queue up behind each other)
    __shared__ uint32_t part[4][kFilterTQ];
#pragma unroll
    for (int t = 0; t < kFilterTQ; ++t) {
        uint32_t v = local[t];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += (uint32_t)__shfl_xor((int)v, off, 64);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6][t] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < nvq) {
        const unsigned long long v = (unsigned long long)part[0][threadIdx.x] + part[1][threadIdx.x] +
                                     part[2][threadIdx.x] + part[3][threadIdx.x];
        if (v) atomicAdd(&nsurv[q0 + threadIdx.x], v);
    }
}

template <int M>
__global__ void __launch_bounds__(256)
hamming_histogram_kernel(const uint8_t *__restrict__ qcodes, const uint8_t *__restrict__ codes, int64_t n,
                         unsigned long long *__restrict__ hist)
{
    constexpr int NB = 8 * M + 1;
    __shared__ unsigned int wbins[4][NB];  // one set of bins per wave: fewer lanes fight over a counter
    unsigned int *bins = wbins[threadIdx.x >> 6];
    const int64_t q = blockIdx.y;
    constexpr int WPC = M / 4;
    for (int b = threadIdx.x; b < 4 * NB; b += 256) (&wbins[0][0])[b] = 0u;
    uint32_t qw[WPC];
#pragma unroll
    for (int w = 0; w < WPC; ++w) qw[w] = ((const uint32_t *)qcodes)[q * WPC + w];
    __syncthreads();
    // (a workgroup sees fewer than 2^32 codes: the grid has at least n / 2^31 columns)
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        int h = 0;
#pragma unroll
        for (int w = 0; w < WPC; ++w) h += __popc(((const uint32_t *)codes)[i * WPC + w] ^ qw[w]);
        atomicAdd(&bins[h], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < NB; b += 256) {
        const unsigned long long v = (unsigned long long)wbins[0][b] + wbins[1][b] + wbins[2][b] + wbins[3][b];
        if (v) atomicAdd(&hist[b], v);
    }
}

__global__ void zero_u64_kernel(unsigned long long *p, int64_t n)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) p[e] = 0;
}

template <int M, int TQ, int NW, bool IVF, bool SHARE>
int run_scan(const ScanArgs &a, int64_t ntiles, size_t lds, hipStream_t s)
{
    static bool configured = false;  // raise the dynamic-LDS ceiling once per instantiation
    if (!configured) {
        PSC_HIP_TRY(hipFuncSetAttribute((const void *)scan_kernel<M, TQ, NW, IVF, SHARE>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        configured = true;
    }
    hipLaunchKernelGGL((scan_kernel<M, TQ, NW, IVF, SHARE>), dim3((unsigned)ntiles), dim3(NW * 64), lds, s, a);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

template <int NW, bool SHARE, bool IVF = false>
int run_scan_mfma(const ScanArgs &a, int64_t ntiles, size_t lds, hipStream_t s)
{
    static bool configured = false;
    if (!configured) {
        PSC_HIP_TRY(hipFuncSetAttribute((const void *)scan_mfma_kernel<NW, SHARE, IVF>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        configured = true;
    }
    hipLaunchKernelGGL((scan_mfma_kernel<NW, SHARE, IVF>), dim3((unsigned)ntiles), dim3(NW * 64), lds, s, a);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

template <int M, int TQ, int NW, bool SHARE, bool FILTER>
int run_adc(const ScanArgs &a, int64_t ntiles, size_t lds, hipStream_t s)
{
    static bool configured = false;
    if (!configured) {
        PSC_HIP_TRY(hipFuncSetAttribute((const void *)adc_kernel<M, TQ, NW, SHARE, FILTER>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        configured = true;
    }
    hipLaunchKernelGGL((adc_kernel<M, TQ, NW, SHARE, FILTER>), dim3((unsigned)ntiles), dim3(NW * 64), lds, s, a);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

template <bool SHARE, bool FILTER>
int dispatch_adc(int m, int tq, int nwaves, const ScanArgs &a, int64_t ntiles, size_t lds, hipStream_t s)
{
    if constexpr (FILTER) {
        if (m == 8 && tq == 8 && nwaves == 8) return run_adc<8, 8, 8, SHARE, true>(a, ntiles, lds, s);
    }
    if (nwaves != 16) {
        set_error("no kernel for tile shape m=%d tq=%d waves=%d", m, tq, nwaves);
        return PSC_EINVAL;
    }
    if (m == 8) {
        if (tq == 16) return run_adc<8, 16, 16, SHARE, FILTER>(a, ntiles, lds, s);
        if (tq == 8) return run_adc<8, 8, 16, SHARE, FILTER>(a, ntiles, lds, s);
        return run_adc<8, 4, 16, SHARE, FILTER>(a, ntiles, lds, s);
    }
    if (tq == 8) return run_adc<16, 8, 16, SHARE, FILTER>(a, ntiles, lds, s);
    return run_adc<16, 4, 16, SHARE, FILTER>(a, ntiles, lds, s);
}

// Share of uniformly random b-bit codes within Hamming distance ht of a given one: what the
// launcher goes by when it picks the kernel (real codes differ, but not by enough to matter for
// a choice between two kernels that both give the same results).
double random_code_survival(int nbits, int ht)
{
    double c = 1.0, sum = 0.0;  // c = C(nbits, i) / 2^nbits, built up stepwise
    for (int i = 0; i < nbits; ++i) c *= 0.5;
    for (int i = 0; i <= ht && i <= nbits; ++i) {
        sum += c;
        c = c * (double)(nbits - i) / (double)(i + 1);
    }
    return sum;
}

// The tile shapes plan_scan hands out (queries per tile x waves per workgroup).
template <bool IVF, bool SHARE>
int dispatch_scan(int m, int tq, int nwaves, const ScanArgs &a, int64_t ntiles, size_t lds, hipStream_t s)
{
    if constexpr (IVF) {
        if (m == 8 && tq == 4 && nwaves == 8) return run_scan<8, 4, 8, true, SHARE>(a, ntiles, lds, s);
        if (m == 8 && tq == 4 && nwaves == 16) return run_scan<8, 4, 16, true, SHARE>(a, ntiles, lds, s);
        if (m == 16 && tq == 8 && nwaves == 16) return run_scan<16, 8, 16, true, SHARE>(a, ntiles, lds, s);
        if (m == 16 && tq == 4 && nwaves == 16) return run_scan<16, 4, 16, true, SHARE>(a, ntiles, lds, s);
    } else {
        if (m == 8 && tq == 8 && nwaves == 8) return run_scan<8, 8, 8, false, SHARE>(a, ntiles, lds, s);
        if (m == 8 && tq == 16 && nwaves == 16) return run_scan<8, 16, 16, false, SHARE>(a, ntiles, lds, s);
        if (m == 8 && tq == 8 && nwaves == 16) return run_scan<8, 8, 16, false, SHARE>(a, ntiles, lds, s);
        if (m == 8 && tq == 4 && nwaves == 16) return run_scan<8, 4, 16, false, SHARE>(a, ntiles, lds, s);
        if (m == 16 && tq == 8 && nwaves == 16) return run_scan<16, 8, 16, false, SHARE>(a, ntiles, lds, s);
        if (m == 16 && tq == 4 && nwaves == 16) return run_scan<16, 4, 16, false, SHARE>(a, ntiles, lds, s);
    }
    set_error("no kernel for tile shape m=%d tq=%d waves=%d", m, tq, nwaves);
    return PSC_EINVAL;
}

constexpr size_t kLdsBudget = 160 * 1024;

thread_local char g_route[96] = "";

void note_route(const char *kernel, int m, int tq, int nwaves, int nslice, int64_t ntiles)
{
    snprintf(g_route, sizeof g_route, "%s m=%d tq=%d waves=%d slices=%d tiles=%lld", kernel, m, tq, nwaves, nslice,
             (long long)ntiles);
}

}  // namespace

std::atomic<int> g_filter_route{PSC_ROUTE_AUTO};

const char *last_scan_route() { return g_route; }

void note_scan_route(const char *text) { snprintf(g_route, sizeof g_route, "%s", text); }

// Tile shape and database slices.
// Shapes (queries per tile x waves per workgroup), per kind of scan, first one that fits:
//  * fused scan, 64-bit codes, more than 16 queries: 8 x 8, two workgroups per compute unit (one
//    stages its tables or waits on a list lock while the other filters; fewer waves per list
//    lock) -- measured 4% (clustered codes) to 11% (random codes) ahead of 16 x 16 at ht=24;
//    falls back to 16 x 16, 8 x 16, 4 x 16 as k grows (the lists share LDS with the tables);
//  * fused scan with the matrix-core filter (64-bit codes, 9 queries or more, few survivors):
//    16 x 16, the only shape of scan_mfma_kernel (k up to 136);
//  * up to 4 / 8 / 16 queries: no more query slots than queries (every slot costs filter work),
//    which keeps a one-pass scan of few queries bound by memory bandwidth;
//  * grouped inverted-file jobs: 4 x 8, three workgroups per compute unit (tiles are short, so
//    their set-up and tail overlap better: 12.4 -> 9.3 ms on the 100M workload);
//  * dense route, with or without the Hamming test: the 16-wave shapes (70 against 76 ms for
//    8 x 8 at 64 bits).
int plan_scan(int m, int64_t nq, int64_t n, int k, int kind, ScanPlan *plan)
{
    if (m != 8 && m != 16) {
        set_error("m must be 8 or 16, got %d", m);
        return PSC_EINVAL;
    }
    if (k < 1 || k > PSC_MAX_K) {
        set_error("k must be in [1, %d], got %d", PSC_MAX_K, k);
        return PSC_EINVAL;
    }
    if (nq < 0 || n < 0 || n >= ((int64_t)1 << 40)) {
        set_error("bad sizes nq=%lld n=%lld", (long long)nq, (long long)n);
        return PSC_EINVAL;
    }
    ScanPlan p;
    p.kpad = (k + 3) / 4 * 4;
    struct Shape {
        int tq, nwaves;
        size_t max_lds;  // the shape is meant for this many bytes at most (several workgroups per unit)
    };
    const int tq_cap = nq <= 4 ? 4 : (nq <= 8 ? 8 : 16);
    Shape options[5];
    int nopt = 0;
    if (kind == kScanFusedMfma) {
        if (m != 8 || nq < kMfmaMinQueries) {
            set_error("the matrix-core filter takes 64-bit codes and at least %d queries", (int)kMfmaMinQueries);
            return PSC_EINVAL;
        }
        options[nopt++] = Shape{16, 16, kLdsBudget};
    } else {
        if (m == 8 && kind == kScanLists) options[nopt++] = Shape{4, 8, kLdsBudget / 2};
        if (m == 8 && kind == kScanFused && nq > 16)
            options[nopt++] = Shape{8, 8, kLdsBudget / 2};
        if (m == 8 && kind != kScanLists) options[nopt++] = Shape{16, 16, kLdsBudget};
        if (kind != kScanLists || m == 16) options[nopt++] = Shape{8, 16, kLdsBudget};
        options[nopt++] = Shape{4, 16, kLdsBudget};
    }
    p.tq = 0;
    for (int o = 0; o < nopt; ++o) {
        const int t = options[o].tq, nw = options[o].nwaves;
        if (t > tq_cap) continue;
        const size_t need = (size_t)t * m * 256 * 4 + (size_t)t * p.kpad * 8 + (size_t)t * 16 + (size_t)t * m * 5 +
                            (size_t)nw * (kQueueCap + 64) * 4 + (kind == kScanFusedMfma ? kMfmaTableBytes : 0);
        if (need <= options[o].max_lds) {
            p.tq = t;
            p.nwaves = nw;
            p.lds_bytes = need;
            break;
        }
    }
    if (p.tq == 0) {
        set_error("no tile shape fits LDS for m=%d k=%d", m, k);
        return PSC_EINVAL;
    }
    // workgroups of this shape a compute unit holds at a time (LDS, and 32 waves)
    p.wgs_per_cu = (int)std::max<size_t>(1, std::min<size_t>(kLdsBudget / p.lds_bytes, (size_t)(32 / p.nwaves)));
    // (one workgroup per unit already saturates memory for a handful of queries, and every further
    //  slice costs list and merge work: measured best at 256 workgroups for 1 to 128 queries)
    const int64_t round = 256 * (int64_t)(nq <= 16 ? 1 : p.wgs_per_cu);
    const int64_t nqt = (nq + p.tq - 1) / p.tq;
    // Slices: one workgroup per (query tile, slice); the launch runs in rounds of `round`
    // workgroups.  Every slice of a query builds its own list of k, which costs insertions and
    // merge work, so the fewest slices win that keep the compute units busy.
    const int64_t block = 512;  // codes per wave and step, at most (64 lanes x 8 codes)
    const int64_t min_slice = p.nwaves * block;  // at least one block per wave
    const int64_t max_by_size = std::max<int64_t>(1, n / min_slice);
    const int64_t max_slice = kind == kScanFusedMfma ? kMfmaMaxSliceLen : kMaxSliceLen;
    const int64_t wg_limit = std::max<int64_t>(8 * round, nqt);
    int64_t want = 1, tiles_one = 0;
    if (nqt > 0 && nq <= 16) {
        // a handful of queries: score = share of the rounds' places that are used, less 1% per round
        double best_score = -1.0;
        for (int64_t sN = 1; sN * nqt <= wg_limit; ++sN) {
            const int64_t wg = nqt * sN, rounds = (wg + round - 1) / round;
            const double score = (double)wg / (double)(rounds * round) - 0.01 * (double)rounds;
            if (score > best_score + 1e-9) {
                best_score = score;
                want = sN;
            }
        }
    } else if (nqt > 0) {
        // Batches: the query tiles that fill whole rounds are scanned in one piece each, only the
        // tiles of the last, partial round are cut into slices (see flat_tile) -- or all tiles are
        // cut alike, whichever is estimated cheaper.  Time in units of "one workgroup scans the
        // whole database": the whole rounds, plus the rounds of the sliced tiles at 1/S each;
        // every extra list of a query is charged 4% (measured: two lists instead of one for all
        // queries cost about 8% at the headline size).
        double best_cost = 1e300;
        const int64_t whole_rounds_tiles = n <= max_slice ? (nqt / round) * round : 0;
        for (int64_t t1 : {whole_rounds_tiles, (int64_t)0}) {
            const int64_t rest = nqt - t1;
            for (int64_t sN = 1; sN <= std::min<int64_t>(max_by_size, 1024) && rest * sN <= wg_limit; ++sN) {
                const double time = (double)t1 / (double)round +
                                    (rest ? (double)((rest * sN + round - 1) / round) / (double)sN : 0.0);
                const double extra = (double)(rest * (sN - 1)) / (double)nqt;
                const double cost = time * (1.0 + 0.04 * extra);
                if (cost < best_cost - 1e-12) {
                    best_cost = cost;
                    want = sN;
                    tiles_one = t1;
                }
                if (!rest) break;
            }
        }
    }
    int64_t nslice = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, max_by_size), 1024));
    int64_t slice_len = (((n + nslice - 1) / nslice) + block - 1) / block * block;
    if (slice_len > max_slice) {
        slice_len = max_slice;
        nslice = (n + slice_len - 1) / slice_len;
        if (nslice > 1024) {
            set_error("database too large for one scan call");
            return PSC_EINVAL;
        }
    }
    if (slice_len == 0) slice_len = block;
    nslice = std::max<int64_t>(1, (n + slice_len - 1) / slice_len);
    p.nslice = (int)nslice;
    p.slice_len = slice_len;
    p.tiles_one = tiles_one;
    p.ntiles = tiles_one + (nqt - tiles_one) * nslice;
    const size_t dist_bytes = ((size_t)nq * nslice * k * sizeof(float) + 255) / 256 * 256;
    p.part_bytes = dist_bytes + (size_t)nq * nslice * k * sizeof(int64_t);
    // a query cut into many slices exchanges one word per 64th of them (see ScanArgs::pub_slots)
    p.pub_slots = shared_threshold_words(nslice);
    p.gthr_bytes = ((size_t)nq * p.pub_slots * sizeof(uint32_t) + 255) / 256 * 256;
    p.total_bytes = 256 + p.gthr_bytes + p.part_bytes;
    *plan = p;
    return PSC_OK;
}

int merge_partial_lists(const float *part_d, const int64_t *part_i, int64_t nq, int nlists, int k, const int *status,
                        int64_t *ids, float *dists, hipStream_t s)
{
    return launch_merge(part_d, part_i, nq, nlists, k, status, ids, dists, s);
}

int shared_threshold_words(int64_t lists_per_query)
{
    return lists_per_query >= kManySlices ? (int)std::min<int64_t>(lists_per_query, 64) : 1;
}

size_t flat_scan_workspace_bytes(int m, int64_t nq, int64_t n, int k)
{
    size_t bytes = 0;
    for (int kind : {kScanFused, kScanDense, kScanDenseFiltered}) {
        ScanPlan p;
        if (plan_scan(m, nq, n, k, kind, &p) != PSC_OK) return 0;
        bytes = std::max(bytes, p.total_bytes);
    }
    ScanPlan p;  // the matrix-core route where it applies (it has shapes and slices of its own)
    if (m == 8 && nq >= kMfmaMinQueries && plan_scan(m, nq, n, k, kScanFusedMfma, &p) == PSC_OK)
        bytes = std::max(bytes, p.total_bytes);
    return bytes;
}

// The exchange between the lists of one query (ScanArgs::pub_slots), for `slots` words per query.
static void set_exchange(ScanArgs &a, int slots, int k)
{
    a.pub_slots = slots;
    a.pub_r = k;
    a.pub_kth = 1;
    if (slots > 1) {
        a.pub_r = std::min(k, std::max(1, (5 * k + 2 * slots - 1) / (2 * slots)));
        a.pub_kth = (k + a.pub_r - 1) / a.pub_r;
    }
}

int launch_scan(int m, const float *lut_dev, const uint8_t *qcodes_dev, int64_t nq,
                const uint8_t *codes_dev, int64_t n, int ht, int k, int64_t skip_first,
                bool clear_status, int64_t *ids_dev, float *dists_dev, void *ws, size_t ws_bytes,
                hipStream_t s)
{
    PSC_REQUIRE(ht >= 0, "ht must be >= 0, got %d", ht);
    // survivor share from which scoring every pair is the faster route: the dense kernel takes the
    // same time whatever the threshold (it tests only the pairs that beat the k-th best), the fused
    // one grows with the survivors (measured at 10M x 10k random codes, fused / dense: 64-bit codes
    // ht = 29: 67.8 / 68.5 ms, ht = 30: 83.1 / 68.6; 128-bit codes ht = 60: 112 / 135, ht = 62: 152 / 135)
    const double dense_from = 0.34;
    const bool dense = ht >= 8 * m || random_code_survival(8 * m, ht) >= dense_from;
    ScanPlan p;
    int rc = PSC_EINVAL;
    // Matrix-core filter: 64-bit codes, more than one tile of queries, k small enough for its
    // 16-query tile, and few survivors (beyond about one pair in ten the queue and the lists
    // decide the time and the two filters tie: measured equal at ht = 26, behind at ht = 28).
    // psc_set_filter_route overrides the rule (for measurements).
    bool mfma = !dense && m == 8 && nq >= kMfmaMinQueries && random_code_survival(8 * m, ht) < 0.10;
    const int forced = g_filter_route.load(std::memory_order_relaxed);
    if (forced == PSC_ROUTE_POPCOUNT) mfma = false;
    if (forced == PSC_ROUTE_MFMA) mfma = !dense && m == 8 && nq >= kMfmaMinQueries;
    if (mfma) {
        rc = plan_scan(m, nq, n, k, kScanFusedMfma, &p);
        mfma = rc == PSC_OK;  // (k too large for the shape: the popcount kernel's shapes take over)
    }
    if (!mfma)
        rc = plan_scan(m, nq, n, k, !dense ? kScanFused : (ht >= 8 * m ? kScanDense : kScanDenseFiltered), &p);
    if (rc != PSC_OK) return rc;
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(ids_dev && dists_dev, "null result pointer");
    if (n == 0) {
        const int64_t total = nq * k;
        hipLaunchKernelGGL(fill_padding_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           ids_dev, dists_dev, total);
        PSC_HIP_TRY(hipGetLastError());
        return PSC_OK;
    }
    PSC_REQUIRE(lut_dev && qcodes_dev && codes_dev, "null input pointer");
    PSC_REQUIRE(((uintptr_t)codes_dev & 15) == 0 && ((uintptr_t)qcodes_dev & 15) == 0 &&
                    ((uintptr_t)lut_dev & 15) == 0,
                "codes, query codes and tables must be 16-byte aligned");
    PSC_REQUIRE(ws && ws_bytes >= p.total_bytes, "workspace too small: need %zu bytes, got %zu",
                p.total_bytes, ws_bytes);
    PSC_REQUIRE(((uintptr_t)ws & 255) == 0, "workspace must be 256-byte aligned");
    PSC_REQUIRE(p.ntiles <= 0x7fffffffLL, "too many tiles");

    ScanArgs a;
    a.lut = lut_dev;
    a.qcodes = qcodes_dev;
    a.codes = codes_dev;
    a.skip_first = skip_first;
    a.nq = nq;
    a.n = n;
    a.slice_len = p.slice_len;
    a.nslice = p.nslice;
    a.tiles_one = p.tiles_one;
    a.k = k;
    a.kpad = p.kpad;
    const int nbits = 8 * m;
    const int ht_eff = ht > nbits ? nbits : ht;
    a.bias = 0x7fffffffu - (uint32_t)ht_eff;
    a.status = (int *)ws;
    a.gthr = (uint32_t *)((char *)ws + 256);
    a.job_q = nullptr;
    a.part_d = (float *)((char *)ws + 256 + p.gthr_bytes);
    a.part_i = (int64_t *)((char *)a.part_d + (((size_t)nq * p.nslice * k * sizeof(float) + 255) / 256 * 256));
    // which entry the lists of a many-slice query publish, and which of the published values bounds
    // the k-th best: pub_kth words x pub_r entries >= k, with pub_kth about 0.4 of the words (the
    // value then sits near the (1.3 k)-th best of everything scanned so far)
    set_exchange(a, p.pub_slots, k);
    const int64_t nwords = nq * p.pub_slots;
    hipLaunchKernelGGL(init_scan_kernel, dim3((unsigned)((nwords + 255) / 256)), dim3(256), 0, s, a.gthr, nwords,
                       clear_status ? a.status : (int *)nullptr);
    // A single query leaves three of the narrowest tile's four query slots empty: they take copies of
    // its tables and code, every wave feeds the list of slot wave % 4, and the four lists are merged
    // when the slice ends -- a list's lock is then shared by 4 waves instead of 16 while the lists
    // fill.
    a.spread_lists = (nq == 1 && skip_first < 0) ? 1 : 0;
    a.list_tab = nullptr;
    a.queries = nullptr;
    a.coarse = nullptr;
    a.job_qcodes = nullptr;
    a.dim = 0;
    a.nlist = 0;
    a.tiles = nullptr;
    a.ntiles = nullptr;
    a.list_off = nullptr;
    a.ext_ids = nullptr;
    a.job_slot = nullptr;
    if (ht >= nbits)  // nothing to filter: the pure-ADC kernel
        rc = p.nslice >= 4 ? dispatch_adc<true, false>(m, p.tq, p.nwaves, a, p.ntiles, p.lds_bytes, s)
                           : dispatch_adc<false, false>(m, p.tq, p.nwaves, a, p.ntiles, p.lds_bytes, s);
    else if (dense)
        rc = p.nslice >= 4 ? dispatch_adc<true, true>(m, p.tq, p.nwaves, a, p.ntiles, p.lds_bytes, s)
                           : dispatch_adc<false, true>(m, p.tq, p.nwaves, a, p.ntiles, p.lds_bytes, s);
    else if (mfma)
        rc = p.nslice >= 4 ? run_scan_mfma<16, true>(a, p.ntiles, p.lds_bytes, s)
                           : run_scan_mfma<16, false>(a, p.ntiles, p.lds_bytes, s);
    else
        rc = p.nslice >= 4 ? dispatch_scan<false, true>(m, p.tq, p.nwaves, a, p.ntiles, p.lds_bytes, s)
                           : dispatch_scan<false, false>(m, p.tq, p.nwaves, a, p.ntiles, p.lds_bytes, s);
    if (rc != PSC_OK) return rc;
    note_route(ht >= nbits ? "adc_kernel" : dense ? "adc_kernel+filter" : mfma ? "scan_mfma_kernel" : "scan_kernel",
               m, p.tq, p.nwaves, p.nslice, p.ntiles);
    return launch_merge(a.part_d, a.part_i, nq, p.nslice, k, a.status, ids_dev, dists_dev, s);
}

// Which filter the grouped inverted-file scan takes.  The matrix-core kernel needs 64-bit codes,
// k small enough for its 16-job tile, lists within its position field and enough jobs per list
// to fill its tiles (a tile costs the same filter work whether 16 or 4 of its slots are taken).
// It pays only while next to nothing survives the test: its one 16-wave workgroup per compute
// unit cannot overlap one tile's set-up and list work with another tile's filtering as three
// 8-wave workgroups do, and a list is 24k codes, not 10M.  Measured on 100M vectors / 4096 lists
// / 10k queries x 64 probes, k = 100, whole search, xor/popcount against matrix cores:
// ht = 0: 5.2 / 4.5 ms, 16: 5.4 / 4.9, 20: 7.1 / 9.0, 24: 8.6 / 10.5 (k = 1: 6.2 / 6.2).
// Hence thresholds that let fewer than one random pair in 10^4 through (ht <= 17).
// psc_set_filter_route overrides the rule where the kernel can run at all.
bool ivf_scan_on_matrix_cores(int m, int ht, int k, int64_t njobs, int nlist, int64_t max_list_len, ScanPlan *plan)
{
    if (m != 8 || ht >= 64 || max_list_len > kMfmaMaxSliceLen || njobs < kMfmaMinQueries) return false;
    bool take = njobs >= 12 * (int64_t)nlist && random_code_survival(64, ht) < 1e-4;
    const int forced = g_filter_route.load(std::memory_order_relaxed);
    if (forced == PSC_ROUTE_POPCOUNT) take = false;
    if (forced == PSC_ROUTE_MFMA) take = true;
    if (!take) return false;
    ScanPlan p;
    if (plan_scan(m, njobs, max_list_len, k, kScanFusedMfma, &p) != PSC_OK) return false;  // (k too large)
    *plan = p;
    return true;
}

// Inverted-file scan: one workgroup per tile descriptor (up to `max_tiles`; the actual count is
// read on the device), partial lists written at job_slot[job] * k, then one merge per query
// over its nprobe partial lists.
int launch_ivf_scan(int m, int tq, int nwaves, int kpad, size_t lds_bytes, const float *lut_dev,
                    const float *list_tab_dev,
                    const float *queries_dev, const float *coarse_dev, int dim, int nlist,
                    uint8_t *job_qcodes_dev, const uint8_t *codes_dev, int64_t n, int ht, int k,
                    const void *tiles_dev, const int *ntiles_dev, int64_t max_tiles,
                    const int64_t *list_off_dev, const int32_t *ext_ids_dev, const int32_t *job_slot_dev,
                    const int32_t *job_q_dev, uint32_t *gthr_dev, float *part_d, int64_t *part_i, int *status,
                    int64_t nq, int nprobe, int64_t *ids_dev, float *dists_dev, bool on_matrix_cores,
                    bool one_job_per_tile, hipStream_t s)
{
    PSC_REQUIRE(((uintptr_t)codes_dev & 15) == 0 && ((uintptr_t)job_qcodes_dev & 15) == 0 &&
                    ((uintptr_t)lut_dev & 15) == 0 && ((uintptr_t)list_tab_dev & 15) == 0,
                "codes, query codes and tables must be 16-byte aligned");
    PSC_REQUIRE(max_tiles <= 0x7fffffffLL, "too many tiles");
    PSC_REQUIRE(dim % m == 0, "dim must be a multiple of m");
    ScanArgs a;
    a.lut = lut_dev;
    a.qcodes = nullptr;
    a.list_tab = list_tab_dev;
    a.queries = queries_dev;
    a.coarse = coarse_dev;
    a.job_qcodes = job_qcodes_dev;
    a.dim = dim;
    a.nlist = nlist;
    a.codes = codes_dev;
    a.skip_first = -1;
    a.nq = 0;
    a.n = n;
    a.slice_len = 0;
    a.nslice = 1;
    a.tiles_one = 0;
    a.k = k;
    a.kpad = kpad;
    const int nbits = 8 * m;
    a.bias = 0x7fffffffu - (uint32_t)(ht > nbits ? nbits : ht);
    a.part_d = part_d;
    a.part_i = part_i;
    a.status = status;
    a.tiles = (const IvfTile *)tiles_dev;
    a.ntiles = ntiles_dev;
    a.list_off = list_off_dev;
    a.ext_ids = ext_ids_dev;
    a.job_slot = job_slot_dev;
    a.job_q = job_q_dev;
    a.gthr = gthr_dev;
    a.spread_lists = one_job_per_tile ? 1 : 0;
    // Tiles of one job each all start together and warm up side by side: they exchange as the
    // slices of a flat scan do.  Grouped tiles of a large batch run one after the other; there a
    // job mostly inherits the k-th best of the query's nearest lists, which one word carries, and
    // reading more than that on every change of a list costs more than it prunes (measured on 100M
    // vectors, 10k queries x 64 probes: 8.3 ms with one word, 21.9 ms with 64).
    set_exchange(a, one_job_per_tile ? shared_threshold_words(nprobe) : 1, k);  // (gthr_dev holds that many words per query)
    const int64_t nwords = nq * a.pub_slots;
    hipLaunchKernelGGL(init_scan_kernel, dim3((unsigned)((nwords + 255) / 256)), dim3(256), 0, s, gthr_dev, nwords,
                       a.status);
    if (max_tiles > 0) {
        int rc;
        if (on_matrix_cores) {
            PSC_REQUIRE(m == 8 && tq == 16 && nwaves == 16, "the matrix-core scan has one tile shape");
            rc = run_scan_mfma<16, true, true>(a, max_tiles, lds_bytes, s);
        } else {
            rc = dispatch_scan<true, true>(m, tq, nwaves, a, max_tiles, lds_bytes, s);
        }
        if (rc != PSC_OK) return rc;
    }
    note_route(on_matrix_cores ? (list_tab_dev ? "scan_mfma_kernel+lists" : "scan_mfma_kernel+lists+direct-tables")
                               : (list_tab_dev ? "scan_kernel+lists" : "scan_kernel+lists+direct-tables"),
               m, tq, nwaves, 1, max_tiles);
    return launch_merge(part_d, part_i, nq, nprobe, k, status, ids_dev, dists_dev, s);
}

int launch_hamming_filter(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                          int64_t n, int ht, int64_t *nsurv_dev, uint8_t *hdist_dev, hipStream_t s)
{
    if (m != 8 && m != 16) {
        set_error("m must be 8 or 16, got %d", m);
        return PSC_EINVAL;
    }
    PSC_REQUIRE(nq >= 0 && n >= 0 && ht >= 0, "bad sizes");
    if (nq == 0) return PSC_OK;
    PSC_REQUIRE(nsurv_dev && qcodes_dev, "null pointer");
    PSC_REQUIRE(nq <= 65535 * (int64_t)kFilterTQ, "too many queries for one filter call");
    hipLaunchKernelGGL(zero_u64_kernel, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, s,
                       (unsigned long long *)nsurv_dev, nq);
    if (n == 0) return PSC_OK;
    PSC_REQUIRE(codes_dev, "null pointer");
    PSC_REQUIRE(((uintptr_t)codes_dev & 3) == 0 && ((uintptr_t)qcodes_dev & 3) == 0, "codes must be 4-byte aligned");
    const unsigned gx = (unsigned)std::min<int64_t>((n + 255) / 256, 1024);
    const unsigned gy = (unsigned)((nq + kFilterTQ - 1) / kFilterTQ);
    if (m == 8)
        hipLaunchKernelGGL((hamming_filter_kernel<8>), dim3(gx, gy), dim3(256), 0, s, qcodes_dev, nq,
                           codes_dev, n, ht, (unsigned long long *)nsurv_dev, hdist_dev);
    else
        hipLaunchKernelGGL((hamming_filter_kernel<16>), dim3(gx, gy), dim3(256), 0, s, qcodes_dev, nq,
                           codes_dev, n, ht, (unsigned long long *)nsurv_dev, hdist_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

int launch_hamming_histogram(int m, const uint8_t *qcodes_dev, int64_t nq, const uint8_t *codes_dev,
                             int64_t n, int64_t *hist_dev, hipStream_t s)
{
    if (m != 8 && m != 16) {
        set_error("m must be 8 or 16, got %d", m);
        return PSC_EINVAL;
    }
    PSC_REQUIRE(nq >= 0 && n >= 0 && hist_dev, "bad sizes or null histogram");
    PSC_REQUIRE(nq <= 65535, "at most 65535 queries per histogram call");
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(256), 0, s, (unsigned long long *)hist_dev, (int64_t)(8 * m + 1));
    if (nq == 0 || n == 0) return PSC_OK;
    PSC_REQUIRE(qcodes_dev && codes_dev, "null pointer");
    PSC_REQUIRE(((uintptr_t)codes_dev & 3) == 0 && ((uintptr_t)qcodes_dev & 3) == 0, "codes must be 4-byte aligned");
    // (64k codes or more per workgroup: every workgroup ends with up to 8m + 1 global additions)
    const unsigned gx = (unsigned)std::max<int64_t>(std::min<int64_t>((n + 65535) / 65536, 2048), (n >> 31) + 1);
    if (m == 8)
        hipLaunchKernelGGL((hamming_histogram_kernel<8>), dim3(gx, (unsigned)nq), dim3(256), 0, s, qcodes_dev,
                           codes_dev, n, (unsigned long long *)hist_dev);
    else
        hipLaunchKernelGGL((hamming_histogram_kernel<16>), dim3(gx, (unsigned)nq), dim3(256), 0, s, qcodes_dev,
                           codes_dev, n, (unsigned long long *)hist_dev);
    PSC_HIP_TRY(hipGetLastError());
    return PSC_OK;
}

}  // namespace psc
