// Decoder: g <- peeling_decompress(index, count_sketch) of Algorithm 1 (section 2.2).
//
// One workgroup per sketch partition.  The partition's unknowns are the set bits of the
// merged Index in [bounds[a], bounds[a+1]); its 3*m_sub cells and their degrees live in
// LDS for the whole peel, so the rounds cost no HBM traffic and no kernel launches.
//
// Peeling is round-synchronous: in a round every unresolved unknown that touches a cell
// of degree 1 takes its value from the smallest such hash function, reading the sketch
// as it stood when the round began; then all unknowns taken in the round subtract
// themselves from their three cells.  The first round that takes nothing ends the peel.
// Unknowns left over are reported with value 0 and counted.
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

__device__ inline uint32_t deg_of(const uint32_t *deg2, uint32_t c)
{
    return (deg2[c >> 1] >> (16 * (c & 1))) & 0xFFFFu;
}

__global__ void __launch_bounds__(kDecodeThreads)
decode_kernel(const uint32_t *__restrict__ bitmap, const float *__restrict__ sketch,
              const uint32_t *__restrict__ header, const uint32_t *__restrict__ bounds,
              uint32_t *idx_out, float *__restrict__ val_out, float *__restrict__ dense_out,
              uint32_t *status, uint32_t n_c, uint32_t sw0, uint32_t sw1, uint32_t sw2,
              uint32_t ct_floats, uint32_t deg_words)
{
    extern __shared__ uint32_t lds[];
    float *Ct = reinterpret_cast<float *>(lds);       // [ct_floats] cells, later dense tile
    uint32_t *deg2 = lds + ct_floats;                 // [deg_words] two 16-bit degrees per word
    uint32_t *scratch = deg2 + deg_words;             // [32]
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
    // ---- stage the partition's cells (16-byte loads where the tile is aligned), clear degrees
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
    for (uint32_t c = tid; c < deg_words; c += kDecodeThreads) deg2[c] = 0;
    __syncthreads();  // also orders this workgroup's idx_out stores before the loads below
    const uint16_t *deg16 = reinterpret_cast<const uint16_t *>(deg2);

    // Per-thread state for its unknowns (u = tid + q*1024): the three cell numbers
    // (15 bits each) and sign bits packed into 64 bits, one "resolved" bit, and one
    // 2-bit "taken this round via hash j" code.
    uint64_t pk[kDecodeMaxQ];
#pragma unroll
    for (uint32_t q = 0; q < kDecodeMaxQ; ++q) {
        const uint32_t u = tid + q * kDecodeThreads;
        pk[q] = 0;
        if (u < Pa) {
            const Cells cl = cells_of(idx_out[rho0 + u], m_sub, sw0, sw1, sw2);
            pk[q] = uint64_t(cl.c[0]) | (uint64_t(cl.c[1]) << 15) | (uint64_t(cl.c[2]) << 30) |
                    (uint64_t(cl.neg) << 45);
#pragma unroll
            for (int j = 0; j < 3; ++j) atomicAdd(&deg2[cl.c[j] >> 1], 1u << (16 * (cl.c[j] & 1)));
        }
    }
    __syncthreads();
    PHASE_MARK(1);

    // ---- peel
    uint32_t done = 0, rounds = 0;
    const uint32_t live = Pa > tid ? min(kDecodeMaxQ, (Pa - tid + kDecodeThreads - 1) / kDecodeThreads)
                                   : 0u;
    const uint32_t live_mask = live >= 32 ? 0xFFFFFFFFu : ((1u << live) - 1u);
    while (true) {
        uint32_t code = 0;
        if (done != live_mask) {
#pragma unroll
            for (uint32_t q = 0; q < kDecodeMaxQ; ++q) {
                if (((live_mask & ~done) >> q) & 1u) {
                    // opaque copy: keeps the unpacking inside the round loop (hoisting it
                    // for all 16 unknowns would cost more registers than the kernel has)
                    uint32_t plo = uint32_t(pk[q]), phi = uint32_t(pk[q] >> 32);
                    asm volatile("" : "+v"(plo), "+v"(phi));
                    const uint64_t pq = uint64_t(plo) | (uint64_t(phi) << 32);
                    const uint32_t d0 = deg16[uint32_t(pq) & 0x7FFFu],
                                   d1 = deg16[uint32_t(pq >> 15) & 0x7FFFu],
                                   d2 = deg16[uint32_t(pq >> 30) & 0x7FFFu];
                    const uint32_t c = d0 == 1 ? 1u : (d1 == 1 ? 2u : (d2 == 1 ? 3u : 0u));
                    code |= c << (2 * q);
                }
            }
        }
        // Nothing has been written yet: a cell of degree 1 keeps its value until its
        // own unknown subtracts itself below, so the value can be read there.
        if (!__syncthreads_or(code != 0)) break;
        ++rounds;
        if (code) {
#pragma unroll
            for (uint32_t q = 0; q < kDecodeMaxQ; ++q) {
                const uint32_t c = (code >> (2 * q)) & 3u;
                if (c) {
                    uint32_t plo = uint32_t(pk[q]), phi = uint32_t(pk[q] >> 32);
                    asm volatile("" : "+v"(plo), "+v"(phi));
                    const uint64_t pq = uint64_t(plo) | (uint64_t(phi) << 32);
                    const uint32_t cc[3] = {uint32_t(pq) & 0x7FFFu, uint32_t(pq >> 15) & 0x7FFFu,
                                            uint32_t(pq >> 30) & 0x7FFFu};
                    const uint32_t neg = uint32_t(pq >> 45) & 7u;
                    const uint32_t j = c - 1;
                    const float cv = Ct[j == 0 ? cc[0] : (j == 1 ? cc[1] : cc[2])];
                    const float x = ((neg >> j) & 1u) ? -cv : cv;
                    val_out[rho0 + tid + q * kDecodeThreads] = x;
#pragma unroll
                    for (int jj = 0; jj < 3; ++jj) {
                        atomicAdd(&Ct[cc[jj]], ((neg >> jj) & 1u) ? x : -x);
                        atomicSub(&deg2[cc[jj] >> 1], 1u << (16 * (cc[jj] & 1)));
                    }
                    done |= 1u << q;
                }
            }
        }
        __syncthreads();
    }

    PHASE_MARK(2);
    // ---- unresolved unknowns get 0; status
    uint32_t unresolved = 0;
#pragma unroll
    for (uint32_t q = 0; q < kDecodeMaxQ; ++q) {
        const uint32_t u = tid + q * kDecodeThreads;
        if (u < Pa && !((done >> q) & 1u)) {
            val_out[rho0 + u] = 0.0f;
            ++unresolved;
        }
    }
    unresolved = block_sum<uint32_t, kDecodeThreads / 64>(unresolved, scratch);
    if (tid == 0) {
        if (unresolved) atomicAdd(&status[TAGC_ST_UNRESOLVED], unresolved);
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

int launch_decode(const tagc_plan_t *p, const tagc_shared_buffers *sh, uint32_t *idx_out,
                  float *val_out, float *dense_out, hipStream_t s)
{
    ProfileScope ps("decode", s);
    const uint32_t ct_floats = std::max<uint32_t>(p->T_cap, 16384);  // cells, or a dense half-tile
    const uint32_t deg_words = p->T_cap / 2 + 1;
    const size_t lds = (size_t(ct_floats) + deg_words + 32) * 4;
    static size_t attr_bytes = 0;
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(decode_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
            return TAGC_EHIP;
        attr_bytes = lds;
    }
    decode_kernel<<<uint32_t(p->A_cap), kDecodeThreads, lds, s>>>(
        sh->bitmap, sh->sketch, sh->header, sh->bounds, idx_out, val_out, dense_out, sh->status,
        uint32_t(p->n_c), p->seed_word[0], p->seed_word[1], p->seed_word[2], ct_floats, deg_words);
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
