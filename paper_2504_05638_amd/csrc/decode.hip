// Decoder: g <- peeling_decompress(index, count_sketch) of Algorithm 1 (section 2.2).
//
// One workgroup per sketch partition.  The partition's unknowns are the set bits of the
// merged Index in [bounds[a], bounds[a+1]); its 3*m_sub cells live in LDS for the whole
// peel, so the rounds cost no HBM traffic and no kernel launches.
//
// Peeling is round-synchronous: in a round every unresolved unknown that touches a cell
// of degree 1 takes its value from the smallest such hash function, reading the sketch
// as it stood when the round began; then all unknowns taken in the round subtract
// themselves from their three cells.  The first round that takes nothing ends the peel.
// Unknowns left over are reported with value 0 and counted.
//
// The rounds are driven by cells, not by polling unknowns.  Besides its value every cell
// keeps one 32-bit word: (sum of the local ranks of its unresolved unknowns) << 15 | degree.
// When the degree is 1 the upper field *is* the remaining unknown, so a queue of the cells
// whose degree has just become 1 is all a round needs; one atomic subtract removes an
// unknown from a cell and tells, by the old degree, whether the cell joins the queue.
// Total work is proportional to the unknowns, not to unknowns x rounds.
#include <type_traits>

#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

// Optional phase timing (build with -DTAGC_PHASE_TIMING): thread 0 of every workgroup
// adds the shader-clock cycles (>> 10) each phase took to status[4 + phase].
#ifdef TAGC_PHASE_TIMING
#define PHASE_MARK(k)                                                        \
    do {                                                                     \
        if (threadIdx.x == 0) {                                              \
            const long long now_ = clock64();                                \
            atomicAdd(&status[4 + (k)], uint32_t((now_ - phase_t0_) >> 10)); \
            phase_t0_ = now_;                                                \
        }                                                                    \
    } while (0)
#define PHASE_INIT() long long phase_t0_ = clock64()
#else
#define PHASE_MARK(k) do { } while (0)
#define PHASE_INIT() do { } while (0)
#endif

constexpr uint32_t kDegMask = 0x7FFFu;  // low 15 bits of a cell's meta word

struct Cells {
    uint32_t c[3];
    uint32_t neg;  // bit j: sign of hash function j is -1
};

__device__ inline Cells cells_of(uint32_t i, uint32_t m_sub, uint32_t sw0, uint32_t sw1,
                                 uint32_t sw2)
{
    Cells r;
    uint32_t n0, n1, n2;
    r.c[0] = hash_slot(i, sw0, m_sub, &n0);
    r.c[1] = m_sub + hash_slot(i, sw1, m_sub, &n1);
    r.c[2] = 2 * m_sub + hash_slot(i, sw2, m_sub, &n2);
    r.neg = n0 | (n1 << 1) | (n2 << 2);
    return r;
}

// Appends `value` to the queue for every active lane with `pred`; one LDS atomic per wave.
__device__ inline void queue_push(bool pred, uint32_t value, uint32_t *count, uint16_t *queue)
{
    const uint64_t bal = __ballot(pred);
    if (bal == 0) return;
    const uint32_t lane = lane_id();
    const uint32_t leader = __builtin_ctzll(bal);
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(count, uint32_t(__popcll(bal)));
    base = __shfl(base, leader, 64);
    if (pred) queue[base + uint32_t(__popcll(bal & ((1ull << lane) - 1ull)))] = uint16_t(value);
}

// Enumerates the set bits of the merged Index in ascending order into idx_out.  One
// workgroup per 1024-word chunk; chunkpre[] (written by the Index aggregation) holds the
// number of set bits before each chunk, so workgroups are independent.  A thread's
// indices are consecutive in the output but a wave's stores, taken entry by entry, would
// hit 64 different cache lines each; so the chunk's first kEnumStage indices are gathered
// in LDS and leave as contiguous stores.
constexpr uint32_t kEnumStage = 8192;

__global__ void __launch_bounds__(256)
enumerate_kernel(const uint32_t *__restrict__ bitmap, uint32_t n_words,
                 const uint32_t *__restrict__ chunkpre, const uint32_t *__restrict__ header,
                 uint32_t *__restrict__ idx_out)
{
    __shared__ uint32_t scratch[8];
    __shared__ uint32_t stage[kEnumStage];
    const uint32_t U = header[TAGC_HDR_U];
    const uint32_t w0 = blockIdx.x * kChunkWords + threadIdx.x * 4;
    uint32_t w[4] = {0, 0, 0, 0};
    if (w0 + 4 <= n_words) {
        const uint4 q = *reinterpret_cast<const uint4 *>(bitmap + w0);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else {
#pragma unroll
        for (uint32_t i = 0; i < 4; ++i) w[i] = w0 + i < n_words ? bitmap[w0 + i] : 0u;
    }
    const uint32_t mine = __popc(w[0]) + __popc(w[1]) + __popc(w[2]) + __popc(w[3]);
    uint32_t tot;
    const uint32_t base = chunkpre[blockIdx.x];
    uint32_t pl = block_excl_scan<uint32_t, 4>(mine, &tot, scratch);  // position in the chunk
#pragma unroll
    for (uint32_t i = 0; i < 4; ++i) {
        uint32_t word = w[i];
        while (word) {
            const uint32_t b = __builtin_ctz(word);
            word &= word - 1;
            const uint32_t v = (w0 + i) * 32 + b;
            if (pl < kEnumStage) stage[pl] = v;
            else if (base + pl < U) idx_out[base + pl] = v;
            ++pl;
        }
    }
    __syncthreads();
    const uint32_t n = min(tot, kEnumStage);
    for (uint32_t i = threadIdx.x; i < n; i += 256)
        if (base + i < U) idx_out[base + i] = stage[i];
}

// Appends up to three values per lane (those whose predicate holds) with one LDS atomic
// per wave; `queue` points at the first free slot of the round, `count` at the number of
// slots the round has taken so far.  Safe in divergent code: only the active lanes take part.
__device__ inline void queue_push3(bool p0, uint32_t v0, bool p1, uint32_t v1, bool p2,
                                   uint32_t v2, uint32_t *count, uint16_t *queue)
{
    const uint64_t b0 = __ballot(p0), b1 = __ballot(p1), b2 = __ballot(p2);
    const uint32_t n0 = __popcll(b0), n1 = __popcll(b1), n2 = __popcll(b2);
    if (n0 + n1 + n2 == 0) return;
    const uint32_t lane = lane_id();
    const uint64_t lt = (1ull << lane) - 1ull;
    const uint32_t leader = __builtin_ctzll(__ballot(true));
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(count, n0 + n1 + n2);
    base = __shfl(base, leader, 64);
    if (p0) queue[base + uint32_t(__popcll(b0 & lt))] = uint16_t(v0);
    if (p1) queue[base + n0 + uint32_t(__popcll(b1 & lt))] = uint16_t(v1);
    if (p2) queue[base + n0 + n1 + uint32_t(__popcll(b2 & lt))] = uint16_t(v2);
}


// One entry of a round's queue: cell q, which had degree 1 when it was queued.  If it still
// has, and its unknown has not been reached through another cell already, the unknown's
// value is read there and taken out of its three cells; cells that thereby reach degree 1
// are queued for the next round.  Called by any subset of a wave's lanes.
__device__ __forceinline__ void resolve_entry(uint32_t q, unsigned long long *cell,
                                              uint32_t *claimed, uint32_t *idx,
                                              uint32_t *any_now, uint32_t *n_next,
                                              uint16_t *next_queue, uint32_t m_sub,
                                              uint32_t sw0, uint32_t sw1, uint32_t sw2)
{
    const unsigned long long oq = cell[q];
    const uint32_t m = uint32_t(oq >> 32);
    if ((m & kDegMask) != 1u) return;  // emptied since it was queued
    const uint32_t u = m >> 15, bit = 1u << (u & 31);
    if (atomicOr(&claimed[u >> 5], bit) & bit) return;  // reached through another cell
    *any_now = 1;
    const Cells cl = cells_of(idx[u], m_sub, sw0, sw1, sw2);
    const uint32_t c[3] = {cl.c[0], cl.c[1], cl.c[2]};
    const uint32_t neg = cl.neg;
    const uint32_t j = c[0] == q ? 0u : (c[1] == q ? 1u : 2u);
    const float cv = __uint_as_float(uint32_t(oq));
    const float x = ((neg >> j) & 1u) ? -cv : cv;
    idx[u] = __float_as_uint(x);  // the c-index has done its job: keep the value there
    const unsigned long long dec = (unsigned long long)((u << 15) + 1u) << 32;
    unsigned long long o[3], r[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) o[k] = uint32_t(k) == j ? oq : cell[c[k]];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const float nv = __uint_as_float(uint32_t(o[k])) + (((neg >> k) & 1u) ? x : -x);
        r[k] = atomicCAS(&cell[c[k]], o[k],
                         ((o[k] - dec) & 0xFFFFFFFF00000000ull) | __float_as_uint(nv));
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        while (r[k] != o[k]) {  // another unknown of the round got there first: redo
            o[k] = r[k];
            const float nv = __uint_as_float(uint32_t(o[k])) + (((neg >> k) & 1u) ? x : -x);
            r[k] = atomicCAS(&cell[c[k]], o[k],
                             ((o[k] - dec) & 0xFFFFFFFF00000000ull) | __float_as_uint(nv));
        }
    }
    queue_push3((uint32_t(o[0] >> 32) & kDegMask) == 2u, c[0],
                (uint32_t(o[1] >> 32) & kDegMask) == 2u, c[1],
                (uint32_t(o[2] >> 32) & kDegMask) == 2u, c[2], n_next, next_queue);
}

// Peels sketch partitions: unknowns rho0 .. rho0+Pa-1 of idx_out, cells a*3*m_sub ...
// An LDS cell is 64 bits: value bits in the low half, meta word (rank-sum << 15 | degree)
// in the high half, so one compare-and-swap subtracts a value and removes an unknown.
//
// The LDS a partition needs leaves room for one workgroup per CU, and the rounds are bound
// by LDS latency, not by memory.  So the grid is one workgroup per CU, each taking
// partitions b, b+G, ...; while one partition is being peeled the cells and c-indices of
// the workgroup's next one are already on their way into registers, and staging it costs
// LDS stores only.
// kCellPre / kIdxPre: cells / unknowns per thread the instantiation can hold (a partition has
// at most kCellPre * kDecodeThreads cells, so a round's queue needs kCellPre sweeps at most).
template <uint32_t kCellPre, uint32_t kIdxPre>
__global__ void __launch_bounds__(kDecodeThreads)
peel_kernel(const float *__restrict__ sketch, const uint32_t *__restrict__ header,
            const uint32_t *__restrict__ idx_out, float *__restrict__ val_out,
            uint32_t *status, uint64_t seed, const uint32_t *__restrict__ salt, uint32_t T_cap,
            uint32_t P_cap, uint32_t mode)
{
    extern __shared__ uint64_t lds64[];
    unsigned long long *cell = reinterpret_cast<unsigned long long *>(lds64);  // [T_cap]
    uint32_t *idx = reinterpret_cast<uint32_t *>(cell + T_cap);      // [P_cap] c-indices
    uint32_t *claimed = idx + P_cap;                 // [P_cap/32 + 1] resolved unknowns
    uint32_t *scratch = claimed + (P_cap / 32 + 1);  // [32]
    uint16_t *queue = reinterpret_cast<uint16_t *>(scratch + 32);  // [T_cap] cells of degree 1
    // Per round: the number of cells the round queued for the next one, and whether it
    // resolved anything.  Three of each, used in turn: round r reads what round r-1 left
    // in slot r%3 (n) resp. (r-1)%3 (any) and writes slot (r+1)%3 resp. r%3, so a wave that
    // is late into round r never sees what faster waves of the same round already write;
    // the slot nobody touches in round r is cleared by thread 0 for its next use.
    __shared__ uint32_t s_n[3], s_any[3];
    const uint32_t tid = threadIdx.x;
    const uint32_t U = header[TAGC_HDR_U], A = header[TAGC_HDR_A];
    const uint32_t m_sub = header[TAGC_HDR_MSUB];
    const uint32_t *meta_hi = reinterpret_cast<const uint32_t *>(cell) + 1;  // meta of cell c: [2c]
    const uint32_t cells = 3 * m_sub;

    // the cells and c-indices of partition `p` into registers (zeros beyond their ends)
    float pre_cell[kCellPre];
    uint32_t pre_idx[kIdxPre];
    auto prefetch = [&](uint32_t p) {
        const uint32_t r0 = uint32_t(uint64_t(p) * U / A);
        const uint32_t n = uint32_t(uint64_t(p + 1) * U / A) - r0;
        const float *src = sketch + uint64_t(p) * cells;
#pragma unroll
        for (uint32_t q = 0; q < kCellPre; ++q) {
            const uint32_t c = tid + q * kDecodeThreads;
            pre_cell[q] = c < cells ? __builtin_nontemporal_load(src + c) : 0.0f;
        }
#pragma unroll
        for (uint32_t q = 0; q < kIdxPre; ++q) {
            const uint32_t u = tid + q * kDecodeThreads;
            pre_idx[q] = u < n ? __builtin_nontemporal_load(idx_out + r0 + u) : 0u;
        }
    };
    if (blockIdx.x < A) prefetch(blockIdx.x);

    uint32_t max_rounds = 0;
    for (uint32_t a = blockIdx.x; a < A; a += gridDim.x) {
    PHASE_INIT();
    const uint32_t rho0 = uint32_t(uint64_t(a) * U / A);
    const uint32_t Pa = uint32_t(uint64_t(a + 1) * U / A) - rho0;
    // the partition's hash functions: the seed under the salt the encoders used
    const uint32_t sa = salt[a];
    const uint32_t sw0 = seed_word(seed, 3 * sa), sw1 = seed_word(seed, 3 * sa + 1),
                   sw2 = seed_word(seed, 3 * sa + 2);

    // ---- stage the partition's cells from the registers, clear state
#pragma unroll
    for (uint32_t q = 0; q < kCellPre; ++q) {
        const uint32_t c = tid + q * kDecodeThreads;
        if (c < cells) cell[c] = __float_as_uint(pre_cell[q]);
    }
    for (uint32_t c = tid; c < P_cap / 32 + 1; c += kDecodeThreads) claimed[c] = 0;
    if (tid < 3) s_n[tid] = s_any[tid] = 0;
    __syncthreads();
    PHASE_MARK(0);

    // ---- every unknown joins its three cells; all values start at 0
#pragma unroll
    for (uint32_t q = 0; q < kIdxPre; ++q) {
        const uint32_t u = tid + q * kDecodeThreads;
        if (u < Pa) {
            const uint32_t i = pre_idx[q];
            idx[u] = i;
            const Cells cl = cells_of(i, m_sub, sw0, sw1, sw2);
            const unsigned long long inc = (unsigned long long)((u << 15) + 1u) << 32;
#pragma unroll
            for (int j = 0; j < 3; ++j) atomicAdd(&cell[cl.c[j]], inc);
        }
    }
    // the registers are free again: the next partition's data travels during the rounds
    if (a + gridDim.x < A) prefetch(a + gridDim.x);
    __syncthreads();
    if (mode != TAGC_DECODE_ESTIMATE) {  // estimation alone: the queue stays empty
        for (uint32_t c0 = 0; c0 < cells; c0 += kDecodeThreads) {
            const uint32_t c = c0 + tid;
            queue_push(c < cells && (meta_hi[2 * c] & kDegMask) == 1u, c, &s_n[1], queue);
        }
    }
    PHASE_MARK(1);

    // ---- peel.  One barrier per round: the queue segment [head, tail) holds the cells
    // that reached degree 1 in the previous round.  A cell of degree 1 is touched by its own
    // unknown only, so whoever claims that unknown may read its value there at any time;
    // every other cell is only ever changed by compare-and-swap.  Removals of a round run
    // concurrently with its claims, which changes neither the set of unknowns the round
    // resolves (a cell that reaches degree 1 now is queued for the next round) nor, beyond
    // rounding order, their values.
    uint32_t rounds = 0, head = 0;
    for (uint32_t r = 1;; ++r) {
        __syncthreads();  // queue, counts and cells of the previous round are complete
        const uint32_t cur = r % 3, nxt = (r + 1) % 3, idle = (r + 2) % 3;
        if (s_any[idle]) ++rounds;  // slot (r-1)%3: did round r-1 resolve anything
        const uint32_t tail = head + s_n[cur];
        if (tail == head) break;
        if (tid == 0) {
            s_n[idle] = 0;     // read in round r-1, added to again in round r+1
            s_any[nxt] = 0;    // read in round r-1 (as its idle slot), set again in round r+1
        }
        for (uint32_t e = head + tid; e < tail; e += kDecodeThreads)
            resolve_entry(queue[e], cell, claimed, idx, &s_any[cur], &s_n[nxt], queue + tail,
                          m_sub, sw0, sw1, sw2);
        head = tail;
    }
    PHASE_MARK(2);

    // ---- values leave in one contiguous sweep (stored one by one as they were found they
    // would cost a cache-line access each); unknowns never claimed stay at 0
    // or, when the plan asks for it, the median of their three signed readings of the
    // cells as the rounds left them (idx[u] still holds the c-index of such an unknown)
    for (uint32_t u = tid; u < Pa; u += kDecodeThreads) {
        float x = 0.0f;
        if ((claimed[u >> 5] >> (u & 31)) & 1u) {
            x = __uint_as_float(idx[u]);
        } else if (mode != TAGC_DECODE_PEEL) {
            const Cells cl = cells_of(idx[u], m_sub, sw0, sw1, sw2);
            float r[3];
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const float cv = __uint_as_float(uint32_t(cell[cl.c[j]]));
                r[j] = ((cl.neg >> j) & 1u) ? -cv : cv;
            }
            x = fmaxf(fminf(r[0], r[1]), fminf(fmaxf(r[0], r[1]), r[2]));
        }
        val_out[rho0 + u] = x;
    }
    uint32_t resolved = 0;
    for (uint32_t c = tid; c < P_cap / 32 + 1; c += kDecodeThreads) resolved += __popc(claimed[c]);
    resolved = block_sum<uint32_t, kDecodeThreads / 64>(resolved, scratch);
    if (tid == 0 && resolved < Pa) {
        atomicAdd(&status[TAGC_ST_UNRESOLVED], Pa - resolved);
        if (mode != TAGC_DECODE_PEEL) atomicAdd(&status[TAGC_ST_ESTIMATED], Pa - resolved);
    }
    max_rounds = max(max_rounds, rounds);
    PHASE_MARK(3);
    }  // partitions of this workgroup
    if (tid == 0 && max_rounds) atomicMax(&status[TAGC_ST_ROUNDS], max_rounds);
}

// ------------------------------------------------- sketch sum inside the decoder
//
// Reduce(count_sketch) and peeling_decompress of Algorithm 1 in one kernel, without a summed
// sketch in memory.  The rounds of a partition are bound by dependent LDS accesses and leave
// the memory system idle; adding up the ranks' sketches is bound by memory and leaves
// everything else idle; run one after the other they cost the sum.  Here a workgroup's 16
// waves split up: kLoadWaves of them do nothing but add up, in rank order, the cells of the
// workgroup's *next* partition in their registers (48 cells per thread), while the other
// kPeelWaves peel the current one in LDS as peel_kernel does.  The two groups meet twice per
// partition, at hardware barriers: when the peelers are done with the LDS (the loaders then
// write the summed cells there) and when that is written.  The peelers' own barriers (after
// the unknowns joined their cells, one per round) must not hold up the loaders, which have
// no part in them and may be waiting for memory: they are counted in an LDS word instead
// (peel_barrier).
constexpr uint32_t kLoadWaves = 4, kPeelWaves = kDecodeThreads / 64 - kLoadWaves;
constexpr uint32_t kLoadThreads = kLoadWaves * 64, kPeelThreads = kPeelWaves * 64;
constexpr uint32_t kLoadCells = (kDefaultPartCells + kLoadThreads - 1) / kLoadThreads;  // per thread
constexpr uint32_t kUnit = 16;  // cells of one rank a loader thread requests at a time
static_assert(kLoadCells == 3 * kUnit, "a rank's cells are three units per loader thread");
constexpr uint32_t kPeelIdx = (kDefaultPartUnknowns + kPeelThreads - 1) / kPeelThreads;

// Barrier among the kPeelWaves peeling waves: every wave adds 1 to an LDS word and goes on
// when the word has reached kPeelWaves x (barriers so far).  All waves of a workgroup are
// resident and every peeling wave reaches every such barrier (they branch on the same LDS
// words), so the wait ends.
__device__ inline void peel_barrier(uint32_t *word, uint32_t &expected)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // this wave's LDS accesses are done
    expected += kPeelWaves;
    if (lane_id() == 0) atomicAdd(word, 1u);
    while (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < expected)
        __builtin_amdgcn_s_sleep(1);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__global__ void __launch_bounds__(kDecodeThreads)
sum_peel_kernel(const RankPtrs rp, uint32_t n_in, const uint32_t *__restrict__ header,
                const uint32_t *__restrict__ idx_out, float *__restrict__ val_out,
                uint32_t *status, uint64_t seed, const uint32_t *__restrict__ salt,
                uint32_t T_cap, uint32_t P_cap, uint32_t mode)
{
    extern __shared__ uint64_t lds64[];
    unsigned long long *cell = reinterpret_cast<unsigned long long *>(lds64);  // [T_cap]
    uint32_t *idx = reinterpret_cast<uint32_t *>(cell + T_cap);      // [P_cap] c-indices
    uint32_t *claimed = idx + P_cap;                 // [P_cap/32 + 1] resolved unknowns
    uint32_t *scratch = claimed + (P_cap / 32 + 1);  // [32]
    uint16_t *queue = reinterpret_cast<uint16_t *>(scratch + 32);  // [T_cap] cells of degree 1
    __shared__ uint32_t s_n[3], s_any[3];  // as in peel_kernel
    __shared__ uint32_t s_bar;             // peel_barrier's word
    __shared__ uint32_t s_resolved;        // unknowns the current partition resolved
    const uint32_t tid = threadIdx.x;
    const uint32_t U = header[TAGC_HDR_U], A = header[TAGC_HDR_A];
    const uint32_t m_sub = header[TAGC_HDR_MSUB];
    const uint32_t cells = 3 * m_sub;
    if (tid == 0) s_bar = 0;
    __syncthreads();

    if (tid >= kPeelThreads) {
        // ------------------------------------------------------------ the loaders
        const uint32_t lt = tid - kPeelThreads;
        // rank r's sketch: read from the kernel argument segment (explicit arguments lie
        // there in declaration order at their natural alignment, `rp` first), because
        // indexing the argument with a run-time r would keep all 32 pointers in registers
        // (a pointer made from an integer has no address space the compiler knows: it is
        // declared global here, or every load through it would be a flat one, which can
        // only be waited for all at once)
        typedef __attribute__((address_space(1))) const float *GlobalCells;
        auto rank_sketch = [&](uint32_t r) -> GlobalCells {
            typedef __attribute__((address_space(4))) const uint64_t *KernArg;
            KernArg ka = (KernArg)__builtin_amdgcn_kernarg_segment_ptr();
            (void)rp;
            return (GlobalCells)ka[r];
        };
        float acc[kLoadCells];
        float b0[kUnit], b1[kUnit], b2[kUnit];
        // third t (cells [16 t, 16 t + 16) of this thread's 48) of `src`, a rank's partition.
        // A whole tile of the default size is read from the partition's first cell on, also
        // where the partition is smaller: a rank's sketch buffer has that much room behind
        // its cells (tagc_plan_sizes), and only the partition's own cells are staged.
        auto request = [&](float (&b)[kUnit], GlobalCells src, auto third) {
            constexpr uint32_t t = decltype(third)::value;
#pragma unroll
            for (uint32_t i = 0; i < kUnit; ++i)
                b[i] = __builtin_nontemporal_load(src + lt + (t * kUnit + i) * kLoadThreads);
        };
        // (the fences keep the compiler from moving the requests of later steps up in front
        // of the adds of earlier ones, which it otherwise does until the registers run out)
        auto add_unit = [&](const float (&b)[kUnit], auto third) {
            constexpr uint32_t t = decltype(third)::value;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (uint32_t i = 0; i < kUnit; ++i) acc[t * kUnit + i] += b[i];
            __builtin_amdgcn_sched_barrier(0);
        };
        constexpr std::integral_constant<uint32_t, 0> T0{};
        constexpr std::integral_constant<uint32_t, 1> T1{};
        constexpr std::integral_constant<uint32_t, 2> T2{};
        // the sum of partition `part` over the ranks, in rank order: the three thirds of a
        // rank are in flight while those of the rank before are added
        auto sum_partition = [&](uint32_t part) {
#pragma unroll
            for (uint32_t q = 0; q < kLoadCells; ++q) acc[q] = 0.0f;
            const uint64_t tile = uint64_t(part) * cells;
            GlobalCells src = rank_sketch(0) + tile;
            request(b0, src, T0);
            request(b1, src, T1);
            request(b2, src, T2);
            for (uint32_t r = 1; r < n_in; ++r) {
                src = rank_sketch(r) + tile;
                add_unit(b0, T0); request(b0, src, T0);
                add_unit(b1, T1); request(b1, src, T1);
                add_unit(b2, T2); request(b2, src, T2);
            }
            add_unit(b0, T0);
            add_unit(b1, T1);
            add_unit(b2, T2);
        };
        if (blockIdx.x < A) sum_partition(blockIdx.x);
        for (uint32_t a = blockIdx.x; a < A; a += gridDim.x) {
            __syncthreads();  // the peelers are done with the LDS
#pragma unroll
            for (uint32_t q = 0; q < kLoadCells; ++q) {
                const uint32_t c = lt + q * kLoadThreads;
                if (c < cells) cell[c] = __float_as_uint(acc[q]);
            }
            __syncthreads();  // the partition is staged
            if (a + gridDim.x < A) sum_partition(a + gridDim.x);
        }
        return;
    }

    // ---------------------------------------------------------------- the peelers
    uint32_t *meta_hi = reinterpret_cast<uint32_t *>(cell) + 1;  // meta of cell c: [2c]
    uint32_t pre_idx[kPeelIdx];
    auto prefetch_idx = [&](uint32_t p) {
        const uint32_t r0 = uint32_t(uint64_t(p) * U / A);
        const uint32_t n = uint32_t(uint64_t(p + 1) * U / A) - r0;
#pragma unroll
        for (uint32_t q = 0; q < kPeelIdx; ++q) {
            const uint32_t u = tid + q * kPeelThreads;
            pre_idx[q] = u < n ? __builtin_nontemporal_load(idx_out + r0 + u) : 0u;
        }
    };
    if (blockIdx.x < A) prefetch_idx(blockIdx.x);
    uint32_t bar_expected = 0, max_rounds = 0, Pa_prev = 0;
    for (uint32_t a = blockIdx.x; a < A; a += gridDim.x) {
        const uint32_t rho0 = uint32_t(uint64_t(a) * U / A);
        const uint32_t Pa = uint32_t(uint64_t(a + 1) * U / A) - rho0;
        const uint32_t sa = salt[a];
        const uint32_t sw0 = seed_word(seed, 3 * sa), sw1 = seed_word(seed, 3 * sa + 1),
                       sw2 = seed_word(seed, 3 * sa + 2);
        __syncthreads();  // everybody is done with the previous partition
        if (tid == 0) {
            // what the previous partition left unresolved
            if (a != blockIdx.x && s_resolved < Pa_prev) {
                atomicAdd(&status[TAGC_ST_UNRESOLVED], Pa_prev - s_resolved);
                if (mode != TAGC_DECODE_PEEL)
                    atomicAdd(&status[TAGC_ST_ESTIMATED], Pa_prev - s_resolved);
            }
            s_resolved = 0;
        }
        for (uint32_t c = tid; c < P_cap / 32 + 1; c += kPeelThreads) claimed[c] = 0;
        if (tid < 3) s_n[tid] = s_any[tid] = 0;
        __syncthreads();  // the loaders have staged the cells

        // ---- every unknown joins its three cells
#pragma unroll
        for (uint32_t q = 0; q < kPeelIdx; ++q) {
            const uint32_t u = tid + q * kPeelThreads;
            if (u < Pa) {
                const uint32_t i = pre_idx[q];
                idx[u] = i;
                const Cells cl = cells_of(i, m_sub, sw0, sw1, sw2);
                const unsigned long long inc = (unsigned long long)((u << 15) + 1u) << 32;
#pragma unroll
                for (int j = 0; j < 3; ++j) atomicAdd(&cell[cl.c[j]], inc);
            }
        }
        if (a + gridDim.x < A) prefetch_idx(a + gridDim.x);
        peel_barrier(&s_bar, bar_expected);
        if (mode != TAGC_DECODE_ESTIMATE) {
            for (uint32_t c0 = 0; c0 < cells; c0 += kPeelThreads) {
                const uint32_t c = c0 + tid;
                queue_push(c < cells && (meta_hi[2 * c] & kDegMask) == 1u, c, &s_n[1], queue);
            }
        }

        // ---- the rounds (see peel_kernel)
        uint32_t rounds = 0, head = 0;
        for (uint32_t r = 1;; ++r) {
            peel_barrier(&s_bar, bar_expected);
            const uint32_t cur = r % 3, nxt = (r + 1) % 3, idle = (r + 2) % 3;
            if (s_any[idle]) ++rounds;
            const uint32_t tail = head + s_n[cur];
            if (tail == head) break;
            if (tid == 0) {
                s_n[idle] = 0;
                s_any[nxt] = 0;
            }
            for (uint32_t e = head + tid; e < tail; e += kPeelThreads)
                resolve_entry(queue[e], cell, claimed, idx, &s_any[cur], &s_n[nxt],
                              queue + tail, m_sub, sw0, sw1, sw2);
            head = tail;
        }

        // ---- output (see peel_kernel)
        for (uint32_t u = tid; u < Pa; u += kPeelThreads) {
            float x = 0.0f;
            if ((claimed[u >> 5] >> (u & 31)) & 1u) {
                x = __uint_as_float(idx[u]);
            } else if (mode != TAGC_DECODE_PEEL) {
                const Cells cl = cells_of(idx[u], m_sub, sw0, sw1, sw2);
                float rd[3];
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const float cv = __uint_as_float(uint32_t(cell[cl.c[j]]));
                    rd[j] = ((cl.neg >> j) & 1u) ? -cv : cv;
                }
                x = fmaxf(fminf(rd[0], rd[1]), fminf(fmaxf(rd[0], rd[1]), rd[2]));
            }
            val_out[rho0 + u] = x;
        }
        uint32_t resolved = 0;
        for (uint32_t c = tid; c < P_cap / 32 + 1; c += kPeelThreads) resolved += __popc(claimed[c]);
        resolved = wave_sum(resolved);
        if (lane_id() == 0 && resolved) atomicAdd(&s_resolved, resolved);
        max_rounds = max(max_rounds, rounds);
        Pa_prev = Pa;
    }
    // the last partition's count: every peeling wave has added its share before this barrier
    peel_barrier(&s_bar, bar_expected);
    if (tid == 0) {
        if (blockIdx.x < A && s_resolved < Pa_prev) {
            atomicAdd(&status[TAGC_ST_UNRESOLVED], Pa_prev - s_resolved);
            if (mode != TAGC_DECODE_PEEL) atomicAdd(&status[TAGC_ST_ESTIMATED], Pa_prev - s_resolved);
        }
        if (max_rounds) atomicMax(&status[TAGC_ST_ROUNDS], max_rounds);
    }
}

// Dense output: one workgroup per 1024-word chunk of the Index writes the 32768 floats
// it covers, zeros included.  The chunk's Index words, the number of set bits before each
// word, and the chunk's values (one contiguous run of val_out; its first kDenseStage
// entries, a denser chunk reads the rest one by one) are put in LDS; after that a thread
// builds any four consecutive outputs on its own -- the rank of a set bit is the word's
// count plus a popcount -- so the output goes out in plain contiguous 16-byte stores.
constexpr uint32_t kDenseStage = 8192;

__global__ void __launch_bounds__(kChunkWords)
dense_kernel(const uint32_t *__restrict__ bitmap, uint32_t n_words,
             const uint32_t *__restrict__ chunkpre, const uint32_t *__restrict__ header,
             const float *__restrict__ val_out, float *__restrict__ dense_out)
{
    constexpr uint32_t NT = kChunkWords;  // one thread per Index word of the chunk
    __shared__ uint32_t scratch[NT / 64];
    __shared__ uint32_t s_word[kChunkWords], s_pre[kChunkWords];
    __shared__ float vals[kDenseStage];
    const uint32_t U = header[TAGC_HDR_U];
    const uint32_t tid = threadIdx.x;
    const uint32_t cw0 = blockIdx.x * kChunkWords;  // first word of the chunk
    const uint32_t word = cw0 + tid < n_words ? bitmap[cw0 + tid] : 0u;
    const uint32_t base = chunkpre[blockIdx.x];
    uint32_t tot;
    const uint32_t pre = block_excl_scan<uint32_t, NT / 64>(uint32_t(__popc(word)), &tot, scratch);
    s_word[tid] = word;
    s_pre[tid] = pre;
    const uint32_t n_st = min(tot, kDenseStage);
    for (uint32_t i = tid; i < n_st; i += NT) vals[i] = base + i < U ? val_out[base + i] : 0.f;
    __syncthreads();
    const uint32_t n4 = min(kChunkWords, n_words - cw0) * 8;  // float4 groups of this chunk
    float4 *out = reinterpret_cast<float4 *>(dense_out + uint64_t(cw0) * 32);
    for (uint32_t c = tid; c < n4; c += NT) {
        const uint32_t wd = s_word[c >> 3], sh = (c & 7u) * 4u;
        const uint32_t nib = (wd >> sh) & 0xFu;
        float o[4] = {0.f, 0.f, 0.f, 0.f};
        if (nib) {
            uint32_t r = s_pre[c >> 3] + __popc(wd & ((1u << sh) - 1u));  // rank in the chunk
#pragma unroll
            for (uint32_t b = 0; b < 4; ++b) {
                if ((nib >> b) & 1u) {
                    if (r < kDenseStage) o[b] = vals[r];
                    else if (base + r < U) o[b] = val_out[base + r];
                    ++r;
                }
            }
        }
        st_stream(out + c, make_float4(o[0], o[1], o[2], o[3]));
    }
}

}  // namespace

size_t decode_lds_bytes(uint32_t T_cap, uint32_t P_cap)
{
    return size_t(T_cap) * 8 + (size_t(P_cap) + (P_cap / 32 + 1) + 32) * 4 + size_t(T_cap) * 2 + 16;
}

int launch_decode(const tagc_plan_t *p, const tagc_shared_buffers *sh,
                  const tagc_rank_buffers *ranks, uint32_t n_ranks, uint32_t *idx_out,
                  float *val_out, float *dense_out, hipStream_t s)
{
    // ranks != nullptr: no summed sketch, the decoder adds up the ranks' sketches itself
    const bool fused = ranks != nullptr;
    if (fused && (p->T_cap > kDefaultPartCells || p->P_cap > kDefaultPartUnknowns ||
                  n_ranks > kMaxRanksPerPass))
        return TAGC_EUNSUPPORTED;
    const uint32_t n_words = uint32_t(p->n_c / 32);
    const uint32_t n_chunks = uint32_t(p->n_chunks);
    const uint32_t *chunkpre = static_cast<const uint32_t *>(sh->workspace);
    if (n_chunks) {
        ProfileScope ps("enumerate", s);
        enumerate_kernel<<<n_chunks, 256, 0, s>>>(sh->bitmap, n_words, chunkpre, sh->header,
                                                  idx_out);
    }
    if (fused) {
        ProfileScope ps("sum_peel", s);
        RankPtrs rp{};
        for (uint32_t r = 0; r < n_ranks; ++r) rp.p[r] = ranks[r].sketch;
        const size_t lds = decode_lds_bytes(p->T_cap, p->P_cap);
        uint32_t grid = uint32_t(std::min<uint64_t>(p->A_cap, uint64_t(device_cu_count())));
        if (p->cfg.decode_workgroups) grid = std::min(grid, p->cfg.decode_workgroups);
        static size_t attr_bytes = 0;
        if (lds > attr_bytes) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(sum_peel_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(lds)) != hipSuccess)
                return TAGC_EHIP;
            attr_bytes = lds;
        }
        sum_peel_kernel<<<grid, kDecodeThreads, lds, s>>>(
            rp, n_ranks, sh->header, idx_out, val_out, sh->status, p->cfg.seed,
            sh->bounds + p->A_cap + 1, p->T_cap, p->P_cap, p->cfg.decode_mode);
    } else {
        ProfileScope ps("peel", s);
        const size_t lds = decode_lds_bytes(p->T_cap, p->P_cap);
        // a workgroup takes partitions b, b + grid, ...: any grid size gives the same result
        uint32_t grid = uint32_t(std::min<uint64_t>(p->A_cap, uint64_t(device_cu_count())));
        if (p->cfg.decode_workgroups) grid = std::min(grid, p->cfg.decode_workgroups);
        // the default partition size gets an instantiation that holds exactly its data
        constexpr uint32_t kC0 = (kDefaultPartCells + kDecodeThreads - 1) / kDecodeThreads;
        constexpr uint32_t kI0 = (kDefaultPartUnknowns + kDecodeThreads - 1) / kDecodeThreads;
        constexpr uint32_t kC1 = (kMaxPartCells + kDecodeThreads - 1) / kDecodeThreads;
        constexpr uint32_t kI1 = (kMaxPartUnknowns + kDecodeThreads - 1) / kDecodeThreads;
        const bool small = p->T_cap <= kC0 * kDecodeThreads && p->P_cap <= kI0 * kDecodeThreads;
        auto kernel = small ? peel_kernel<kC0, kI0> : peel_kernel<kC1, kI1>;
        static size_t attr_bytes[2] = {0, 0};
        if (lds > attr_bytes[small]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(lds)) != hipSuccess)
                return TAGC_EHIP;
            attr_bytes[small] = lds;
        }
        kernel<<<grid, kDecodeThreads, lds, s>>>(
            sh->sketch, sh->header, idx_out, val_out, sh->status, p->cfg.seed,
            sh->bounds + p->A_cap + 1, p->T_cap, p->P_cap, p->cfg.decode_mode);
    }
    if (dense_out && n_chunks) {
        ProfileScope ps("dense", s);
        dense_kernel<<<n_chunks, kChunkWords, 0, s>>>(sh->bitmap, n_words, chunkpre, sh->header, val_out,
                                              dense_out);
    }
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
