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
#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

// Optional phase timing (build with -DTAGC_PHASE_TIMING): thread 0 of every workgroup
// adds the shader-clock cycles (>> 10) each phase took to status[3 + phase].
#ifdef TAGC_PHASE_TIMING
#define PHASE_MARK(k)                                                        \
    do {                                                                     \
        if (threadIdx.x == 0) {                                              \
            const long long now_ = clock64();                                \
            atomicAdd(&status[3 + (k)], uint32_t((now_ - phase_t0_) >> 10)); \
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
__device__ inline void queue_push(bool pred, uint32_t value, uint32_t *tail, uint16_t *queue)
{
    const uint64_t bal = __ballot(pred);
    if (bal == 0) return;
    const uint32_t lane = lane_id();
    const uint32_t leader = __builtin_ctzll(bal);
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(tail, uint32_t(__popcll(bal)));
    base = __shfl(base, leader, 64);
    if (pred) queue[base + uint32_t(__popcll(bal & ((1ull << lane) - 1ull)))] = uint16_t(value);
}

__global__ void __launch_bounds__(kDecodeThreads)
decode_kernel(const uint32_t *__restrict__ bitmap, const float *__restrict__ sketch,
              const uint32_t *__restrict__ header, const uint32_t *__restrict__ bounds,
              uint32_t *idx_out, float *val_out, float *__restrict__ dense_out,
              uint32_t *status, uint32_t n_c, uint32_t sw0, uint32_t sw1, uint32_t sw2,
              uint32_t ct_floats, uint32_t T_cap, uint32_t P_cap)
{
    extern __shared__ uint32_t lds[];
    float *Ct = reinterpret_cast<float *>(lds);             // [ct_floats] cells, later dense tile
    uint32_t *meta = lds + ct_floats;                       // [T_cap] rank-sum << 15 | degree
    uint32_t *claimed = meta + T_cap;                       // [P_cap/32 + 1] resolved unknowns
    uint32_t *scratch = claimed + (P_cap / 32 + 1);         // [32]
    uint16_t *queue = reinterpret_cast<uint16_t *>(scratch + 32);  // [T_cap] cells of degree 1
    __shared__ uint32_t s_tail;
    const uint32_t tid = threadIdx.x;
    const uint32_t U = header[TAGC_HDR_U], A = header[TAGC_HDR_A];
    const uint32_t m_sub = header[TAGC_HDR_MSUB];
    const uint32_t a = blockIdx.x;

    if (a >= A) {
        // Empty Index: the dense output is still defined (all zeros); the grid shares it.
        if (A == 0 && dense_out) {
            const uint64_t per = (uint64_t(n_c) + gridDim.x - 1) / gridDim.x;
            const uint64_t lo = per * a, hi = min(uint64_t(n_c), lo + per);
            for (uint64_t i = lo + tid; i < hi; i += kDecodeThreads) dense_out[i] = 0.0f;
        }
        return;
    }

    PHASE_INIT();
    const uint32_t rho0 = uint32_t(uint64_t(a) * U / A);
    const uint32_t Pa = uint32_t(uint64_t(a + 1) * U / A) - rho0;
    const uint32_t ilo = bounds[a], ihi = bounds[a + 1];
    const uint32_t cells = 3 * m_sub;

    // ---- enumerate the set bits of [ilo, ihi) in ascending order into idx_out
    {
        const uint32_t wlo = ilo >> 5, whi = (ihi + 31) >> 5;
        uint32_t running = 0;
        for (uint32_t wb = wlo; wb < whi; wb += kDecodeThreads) {
            const uint32_t w = wb + tid;
            uint32_t word = w < whi ? bitmap[w] : 0u;
            if (w == wlo) word &= 0xFFFFFFFFu << (ilo & 31);
            if ((ihi & 31) && w == (ihi >> 5)) word &= (1u << (ihi & 31)) - 1u;
            uint32_t tot;
            uint32_t pos = running + block_excl_scan<uint32_t, kDecodeThreads / 64>(
                                         uint32_t(__popc(word)), &tot, scratch);
            while (word) {
                const uint32_t b = __builtin_ctz(word);
                word &= word - 1;
                if (pos < Pa) idx_out[rho0 + pos] = w * 32 + b;
                ++pos;
            }
            running += tot;
        }
    }
    PHASE_MARK(0);
    // ---- stage the partition's cells (16-byte loads where the tile is aligned), clear state
    {
        const float *src = sketch + uint64_t(a) * cells;
        const uint32_t head = min(cells, uint32_t((4u - (uint64_t(a) * cells & 3u)) & 3u));
        const uint32_t n4 = (cells - head) / 4;
        if (tid < head) Ct[tid] = src[tid];
        for (uint32_t v = tid; v < n4; v += kDecodeThreads) {
            const float4 q = *reinterpret_cast<const float4 *>(src + head + 4 * v);
            float *d = Ct + head + 4 * v;
            d[0] = q.x; d[1] = q.y; d[2] = q.z; d[3] = q.w;
        }
        for (uint32_t c = head + 4 * n4 + tid; c < cells; c += kDecodeThreads) Ct[c] = src[c];
    }
    for (uint32_t c = tid; c < cells; c += kDecodeThreads) meta[c] = 0;
    for (uint32_t c = tid; c < P_cap / 32 + 1; c += kDecodeThreads) claimed[c] = 0;
    if (tid == 0) s_tail = 0;
    __syncthreads();  // also orders this workgroup's idx_out stores before the loads below

    // ---- every unknown joins its three cells; all values start at 0
    for (uint32_t u = tid; u < Pa; u += kDecodeThreads) {
        const Cells cl = cells_of(idx_out[rho0 + u], m_sub, sw0, sw1, sw2);
#pragma unroll
        for (int j = 0; j < 3; ++j) atomicAdd(&meta[cl.c[j]], (u << 15) + 1u);
        val_out[rho0 + u] = 0.0f;
    }
    __syncthreads();
    for (uint32_t c0 = 0; c0 < cells; c0 += kDecodeThreads) {
        const uint32_t c = c0 + tid;
        queue_push(c < cells && (meta[c] & kDegMask) == 1u, c, &s_tail, queue);
    }
    PHASE_MARK(1);

    // ---- peel
    uint32_t rounds = 0, head = 0;
    while (true) {
        __syncthreads();  // queue and s_tail of the previous phase are complete
        const uint32_t tail = s_tail;
        if (tail == head) break;
        // read phase: claim the unknown of every queued cell that still has degree 1 and
        // fix, from the degrees as they stand now, the hash function its value comes from
        uint32_t mine = 0, jcode = 0;
        for (uint32_t it = 0, e = head + tid; head + it * kDecodeThreads < tail;
             ++it, e += kDecodeThreads) {
            if (e >= tail) continue;
            const uint32_t m = meta[queue[e]];
            if ((m & kDegMask) != 1u) continue;  // emptied later in the round that queued it
            const uint32_t u = m >> 15, bit = 1u << (u & 31);
            if (atomicOr(&claimed[u >> 5], bit) & bit) continue;  // reached through another cell
            const Cells cl = cells_of(idx_out[rho0 + u], m_sub, sw0, sw1, sw2);
            const uint32_t j = (meta[cl.c[0]] & kDegMask) == 1u   ? 0u
                               : (meta[cl.c[1]] & kDegMask) == 1u ? 1u
                                                                  : 2u;
            mine |= 1u << it;
            jcode |= j << (2 * it);
        }
        // barrier between the reads above and the updates below.  A cell of degree 1 is
        // touched by its own unknown only, so its value and rank can still be read there.
        if (!__syncthreads_or(mine != 0)) {
            head = tail;
            continue;
        }
        ++rounds;
        for (uint32_t it = 0; mine >> it; ++it) {
            if (!((mine >> it) & 1u)) continue;
            const uint32_t u = meta[queue[head + it * kDecodeThreads + tid]] >> 15;
            const Cells cl = cells_of(idx_out[rho0 + u], m_sub, sw0, sw1, sw2);
            const uint32_t j = (jcode >> (2 * it)) & 3u;
            const float cv = Ct[j == 0 ? cl.c[0] : (j == 1 ? cl.c[1] : cl.c[2])];
            const float x = ((cl.neg >> j) & 1u) ? -cv : cv;
            val_out[rho0 + u] = x;
#pragma unroll
            for (int jj = 0; jj < 3; ++jj) {
                atomicAdd(&Ct[cl.c[jj]], ((cl.neg >> jj) & 1u) ? x : -x);
                const uint32_t old = atomicSub(&meta[cl.c[jj]], (u << 15) + 1u);
                queue_push((old & kDegMask) == 2u, cl.c[jj], &s_tail, queue);
            }
        }
        head = tail;
    }

    PHASE_MARK(2);
    // ---- status: unknowns never claimed stay at 0
    uint32_t resolved = 0;
    for (uint32_t c = tid; c < P_cap / 32 + 1; c += kDecodeThreads) resolved += __popc(claimed[c]);
    resolved = block_sum<uint32_t, kDecodeThreads / 64>(resolved, scratch);
    if (tid == 0) {
        if (resolved < Pa) atomicAdd(&status[TAGC_ST_UNRESOLVED], Pa - resolved);
        atomicMax(&status[TAGC_ST_ROUNDS], rounds);
    }

    PHASE_MARK(3);
    // ---- dense output: this partition covers c-indices [dlo, ihi).  A second sweep over
    // the Index words: the rank of a word's first set bit (workgroup scan) says where its
    // values sit in val_out, so values are read in order and each tile is written whole.
    if (dense_out) {
        const uint32_t dlo = a == 0 ? 0u : ilo;
        const uint32_t wlo = ilo >> 5;
        uint32_t running = 0;
        __syncthreads();  // val_out stores of this workgroup are read back below
        for (uint32_t wb = dlo >> 5; wb * 32 < ihi; wb += kDecodeThreads) {
            const uint32_t w = wb + tid;
            uint32_t word = (w * 32 < ihi && w >= wlo) ? bitmap[w] : 0u;
            if (w == wlo) word &= 0xFFFFFFFFu << (ilo & 31);
            if ((ihi & 31) && w == (ihi >> 5)) word &= (1u << (ihi & 31)) - 1u;
            uint32_t tot;
            uint32_t pos = running + block_excl_scan<uint32_t, kDecodeThreads / 64>(
                                         uint32_t(__popc(word)), &tot, scratch);
            // the tile of this sweep step: 1024 words = 32768 positions, in two halves
            // of the staging buffer's size
            for (uint32_t half = 0; half < 2; ++half) {
                const uint32_t hbase = (wb + half * 512) * 32;  // first position of the half
                if (hbase >= ihi) break;
                for (uint32_t c = tid; c < 16384; c += kDecodeThreads) Ct[c] = 0.0f;
                __syncthreads();
                if ((tid >> 9) == half) {
                    uint32_t ww = word, pp = pos;
                    while (ww) {
                        const uint32_t bb = __builtin_ctz(ww);
                        ww &= ww - 1;
                        if (pp < Pa) Ct[(tid & 511) * 32 + bb] = val_out[rho0 + pp];
                        ++pp;
                    }
                }
                __syncthreads();
                const uint32_t lo = max(hbase, dlo), hi = min(hbase + 16384, ihi);
                for (uint32_t i = lo + tid; i < hi; i += kDecodeThreads)
                    dense_out[i] = Ct[i - hbase];
                __syncthreads();
            }
            running += tot;
        }
    }
    PHASE_MARK(4);
}

}  // namespace

size_t decode_lds_bytes(uint32_t T_cap, uint32_t P_cap)
{
    const size_t ct_floats = std::max<uint32_t>(T_cap, 16384);  // cells, or a dense half-tile
    return (ct_floats + T_cap + (P_cap / 32 + 1) + 32) * 4 + size_t(T_cap) * 2 + 16;
}

int launch_decode(const tagc_plan_t *p, const tagc_shared_buffers *sh, uint32_t *idx_out,
                  float *val_out, float *dense_out, hipStream_t s)
{
    ProfileScope ps("decode", s);
    const uint32_t ct_floats = std::max<uint32_t>(p->T_cap, 16384);
    const size_t lds = decode_lds_bytes(p->T_cap, p->P_cap);
    static size_t attr_bytes = 0;
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(decode_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
            return TAGC_EHIP;
        attr_bytes = lds;
    }
    decode_kernel<<<uint32_t(p->A_cap), kDecodeThreads, lds, s>>>(
        sh->bitmap, sh->sketch, sh->header, sh->bounds, idx_out, val_out, dense_out, sh->status,
        uint32_t(p->n_c), p->seed_word[0], p->seed_word[1], p->seed_word[2], ct_floats, p->T_cap,
        p->P_cap);
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
