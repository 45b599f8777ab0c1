// Index aggregation: what All-Reduce(local_index) yields in Algorithm 1, computed on one
// GPU as the bitwise OR of N ranks' bit maps (section 2.2 names OR as the operation the
// Index needs), followed by everything the later stages derive from the merged Index:
// its number of non-zeros U, the sketch layout (A partitions of 3*m_sub cells) and the
// c-index at which each partition starts.
#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

// One workgroup per chunk of kChunkWords words of the merged Index; 4 words per thread.
// MODE says how the ranks' wire Indexes combine (section 2.2): the OR the Index needs, or the
// addition that simulates it over a library without OR -- of the 1-bit words themselves
// (carries and all), or of 4-bit counters, four wire words per merged word, a merged bit
// being set where the summed counter is not 0.  Sums wrap as unsigned 32-bit adds do.  With
// more ranks than one launch takes, the running result is carried in `out` (OR, 1-bit add)
// or, for the counters, in `sum4`.
template <int MODE>
__global__ void __launch_bounds__(256)
index_merge_kernel(RankPtrs rp, uint32_t n_in, uint32_t *__restrict__ out, uint32_t n_words,
                   int accumulate, int last, uint32_t *__restrict__ sum4,
                   uint32_t *__restrict__ chunkcnt)
{
    __shared__ uint32_t smem[4];
    const uint32_t w0 = blockIdx.x * kChunkWords + threadIdx.x * 4;
    uint32_t pc = 0;
    if (MODE == TAGC_INDEX_ADD4) {
        // a thread merges the words tid, tid + 256, ... of the chunk: the four wire words of
        // one merged word are one 16-byte load per rank, consecutive across the lanes
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t w = blockIdx.x * kChunkWords + k * 256 + threadIdx.x;
            if (w >= n_words) break;
            const size_t q = 4 * size_t(w);
            uint4 acc = accumulate ? *reinterpret_cast<const uint4 *>(sum4 + q)
                                   : make_uint4(0, 0, 0, 0);
#pragma unroll 8
            for (uint32_t r = 0; r < n_in; ++r) {
                const uint4 v = ld_stream(
                    reinterpret_cast<const uint4 *>(static_cast<const uint32_t *>(rp.p[r]) + q));
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            if (!last) {
                *reinterpret_cast<uint4 *>(sum4 + q) = acc;
            } else {
                const uint32_t m = nibbles_set(acc.x) | (nibbles_set(acc.y) << 8) |
                                   (nibbles_set(acc.z) << 16) | (nibbles_set(acc.w) << 24);
                out[w] = m;
                pc += __popc(m);
            }
        }
    } else if (w0 + 4 <= n_words) {
        uint4 acc = accumulate ? *reinterpret_cast<const uint4 *>(out + w0) : make_uint4(0, 0, 0, 0);
        for (uint32_t r = 0; r < n_in; ++r) {
            const uint4 v =
                ld_stream(reinterpret_cast<const uint4 *>(static_cast<const uint32_t *>(rp.p[r]) + w0));
            if (MODE == TAGC_INDEX_OR1) {
                acc.x |= v.x; acc.y |= v.y; acc.z |= v.z; acc.w |= v.w;
            } else {
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
        }
        *reinterpret_cast<uint4 *>(out + w0) = acc;
        pc = __popc(acc.x) + __popc(acc.y) + __popc(acc.z) + __popc(acc.w);
    } else {
        for (uint32_t w = w0; w < n_words; ++w) {
            uint32_t acc = accumulate ? out[w] : 0u;
            for (uint32_t r = 0; r < n_in; ++r) {
                const uint32_t v = static_cast<const uint32_t *>(rp.p[r])[w];
                acc = MODE == TAGC_INDEX_OR1 ? (acc | v) : (acc + v);
            }
            out[w] = acc;
            pc += __popc(acc);
        }
    }
    if (chunkcnt) {
        pc = block_sum<uint32_t, 4>(pc, smem);
        if (threadIdx.x == 0) chunkcnt[blockIdx.x] = pc;
    }
}

struct LayoutParams {
    uint32_t mode, milli, P_cap, T_cap;
    uint64_t n_real, U_cap, A_cap, m_cap;
};

// Single workgroup: exclusive prefix of the chunk counts (in place, total appended), the
// sketch layout, and a cleared status block.
//
//   target cells  M = ceil(milli*U/1000)  |  ceil(n_real*1000/milli)
//   partitions    A = max(1, ceil(U/P_cap), ceil(M/(3q))),  q = T_cap/3   (0 if U = 0)
//   sub-table     m_sub = max(1, ceil(M/(3A)))  |  max(1, floor(M/(3A)))
//   total         m = 3*A*m_sub
__global__ void __launch_bounds__(1024)
header_kernel(uint32_t *chunk, uint32_t n_chunks, LayoutParams lp, uint32_t *header,
              uint32_t *status)
{
    __shared__ uint32_t smem[16];
    uint32_t running = 0;
    for (uint32_t base = 0; base < n_chunks; base += 1024) {
        const uint32_t i = base + threadIdx.x;
        uint32_t v = i < n_chunks ? chunk[i] : 0u, tot;
        uint32_t ex = block_excl_scan<uint32_t, 16>(v, &tot, smem);
        if (i < n_chunks) chunk[i] = running + ex;
        running += tot;
    }
    if (threadIdx.x != 0) return;
    chunk[n_chunks] = running;
    uint64_t U = running, A = 0, m_sub = 0, m = 0;
    uint32_t flags = 0;
    if (U > 0) {
        uint64_t M = lp.mode == TAGC_SIZE_LOAD_FACTOR ? (uint64_t(lp.milli) * U + 999) / 1000
                                                      : (lp.n_real * 1000 + lp.milli - 1) / lp.milli;
        uint64_t q = lp.T_cap / 3;
        A = (U + lp.P_cap - 1) / lp.P_cap;
        uint64_t A2 = (M + 3 * q - 1) / (3 * q);
        if (A2 > A) A = A2;
        if (A < 1) A = 1;
        m_sub = lp.mode == TAGC_SIZE_LOAD_FACTOR ? (M + 3 * A - 1) / (3 * A) : M / (3 * A);
        if (m_sub < 1) m_sub = 1;
        m = 3 * A * m_sub;
        if (U > lp.U_cap || A > lp.A_cap || m > lp.m_cap) {  // caller broke the plan's bounds
            flags = TAGC_FLAG_OVERFLOW;
            U = A = m_sub = m = 0;
        }
    }
    header[TAGC_HDR_U] = uint32_t(U);
    header[TAGC_HDR_A] = uint32_t(A);
    header[TAGC_HDR_MSUB] = uint32_t(m_sub);
    header[TAGC_HDR_M] = uint32_t(m);
    for (int i = 4; i < TAGC_HDR_WORDS; ++i) header[i] = 0;
    for (int i = 0; i < TAGC_ST_WORDS; ++i) status[i] = 0;
    status[TAGC_ST_FLAGS] = flags;
}

// One wave per partition boundary a: bounds[a] = c-index of the non-zero of rank
// floor(a*U/A); bounds[A] = n_c.
__global__ void __launch_bounds__(256)
bounds_kernel(const uint32_t *__restrict__ bitmap, uint32_t n_words, uint32_t n_c,
              const uint32_t *__restrict__ chunkpre, uint32_t n_chunks,
              const uint32_t *__restrict__ header, uint32_t *__restrict__ bounds)
{
    const uint32_t U = header[TAGC_HDR_U], A = header[TAGC_HDR_A];
    const uint32_t a = blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t l = lane_id();
    if (a > A) return;
    if (a == A) {
        if (l == 0) bounds[a] = n_c;
        return;
    }
    const uint32_t rho = uint32_t(uint64_t(a) * U / A);
    uint32_t lo = 0, hi = n_chunks;  // largest chunk with chunkpre <= rho
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (chunkpre[mid] <= rho) lo = mid; else hi = mid;
    }
    const uint32_t local = rho - chunkpre[lo];
    const uint32_t wbase = lo * kChunkWords + l * 16;
    uint32_t w[16];
    if (wbase + 16 <= n_words) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint4 v = *reinterpret_cast<const uint4 *>(bitmap + wbase + 4 * i);
            w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) w[i] = (wbase + i < n_words) ? bitmap[wbase + i] : 0u;
    }
    uint32_t tot = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot += __popc(w[i]);
    const uint32_t incl = wave_incl_scan<uint32_t>(tot);
    const uint32_t excl = incl - tot;
    if (excl <= local && local < incl) {
        uint32_t r = local - excl;
        uint32_t found = n_c;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t c = __popc(w[i]);
            if (found == n_c) {
                if (r < c) {
                    uint32_t x = w[i];
                    for (uint32_t s = 0; s < r; ++s) x &= x - 1;
                    found = (wbase + i) * 32 + __builtin_ctz(x);
                } else {
                    r -= c;
                }
            }
        }
        bounds[a] = found;
    }
}

// ranges[a] of rank r = number of the rank's pairs whose c-index lies below bounds[a]: the
// pairs of partition a are [ranges[a], ranges[a+1]) of its sorted list.  One thread per
// (rank, boundary); a binary search costs ~20 dependent loads, but all of them run at once
// and the encoder's workgroups, which used to search as they started, no longer wait.
__global__ void __launch_bounds__(256)
ranges_kernel(RankPtrs idx, RankPtrs cnt, uint32_t n_in, const uint32_t *__restrict__ header,
              const uint32_t *__restrict__ bounds, uint32_t A_cap, uint32_t ranges_off,
              uint32_t pair_cap)
{
    const uint32_t A = header[TAGC_HDR_A];
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    const uint32_t r = t / (A_cap + 1), a = t % (A_cap + 1);
    if (r >= n_in || a > A) return;
    uint32_t *c = static_cast<uint32_t *>(const_cast<void *>(cnt.p[r]));
    const uint32_t *ix = static_cast<const uint32_t *>(idx.p[r]);
    const uint32_t n = min(c[TAGC_CNT_TOTAL], pair_cap);
    const uint32_t key = bounds[a];
    uint32_t lo = 0, hi = n;  // first position whose c-index is >= key
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (ix[mid] < key) lo = mid + 1; else hi = mid;
    }
    c[ranges_off + a] = lo;
}

// Per-partition hash salts (the compression is to be lossless, section 2.2 and Table 1).
// Two non-zeros of a partition that fall into the same three cells can never be peeled
// apart, and with the cells of a non-zero confined to its partition that happens to a few
// pairs per 10^8 non-zeros.  The merged Index reaches every rank before compress(g_shard,
// index) runs (Algorithm 1), so encoder and decoder can both derive from it, for every
// partition, the smallest salt under which all of the partition's (slot_0, slot_1, slot_2)
// are distinct; nothing travels.  Nearly every partition keeps salt 0.
//
// One workgroup per partition at a time, two workgroups per compute unit.  The partition's
// non-zeros are the set bits of the merged Index in [bounds[a], bounds[a+1]).  Each gets a
// number t (any order; a wave takes a run of numbers with one LDS add), its three slots under
// the salt being tried, and is pushed on the list of its slot_0 (an LDS exchange of the
// list's head); afterwards it walks what was on that list before it and compares the other
// two slots.  LDS per non-zero: a 32-bit tag (slot_1, slot_2) and a 16-bit link; per cell of
// a sub-table a 32-bit list head -- little enough for two partitions per compute unit, whose
// phases (hashing on the vector units, list building and walking in LDS) then overlap.
constexpr uint32_t kSaltThreads = 1024;
constexpr uint32_t kSaltLimit = 16;       // salts tried: 0 .. 15
constexpr uint32_t kNoLink = 0xFFFFu;
constexpr uint32_t kSaltPre = 4;          // Index words per thread requested a partition ahead

__global__ void __launch_bounds__(kSaltThreads)
salt_kernel(const uint32_t *__restrict__ bitmap, uint32_t n_words,
            const uint32_t *__restrict__ header, const uint32_t *__restrict__ bounds,
            uint32_t *__restrict__ salt_out, uint64_t seed, uint32_t P_cap, uint32_t q_cap)
{
    extern __shared__ uint32_t lds_salt[];
    uint32_t *tag = lds_salt;                        // [P_cap] c-index, then slot_1 | slot_2 << 16
    uint32_t *head = tag + P_cap;                                   // [q_cap]
    uint16_t *link = reinterpret_cast<uint16_t *>(head + q_cap);    // [P_cap]
    __shared__ uint32_t s_n, s_dup;
    const uint32_t A = header[TAGC_HDR_A], m_sub = min(header[TAGC_HDR_MSUB], q_cap);
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    // word `w` of partition [lo, hi), bits outside the partition cleared
    auto load_word = [&](uint32_t w, uint32_t lo, uint32_t hi) -> uint32_t {
        if (lo >= hi || w > ((hi - 1) >> 5) || w >= n_words) return 0u;
        uint32_t word = bitmap[w];
        if (w == (lo >> 5)) word &= 0xFFFFFFFFu << (lo & 31);
        if (w == ((hi - 1) >> 5) && (hi & 31)) word &= (1u << (hi & 31)) - 1u;
        return word;
    };
    // Requests run ahead of the work: the bounds of the partition after the next, and the
    // first Index words of the next one, are on their way while this one is checked.
    uint32_t pre[kSaltPre], lo = 0, hi = 0, lo2 = 0, hi2 = 0;
    const uint32_t G = gridDim.x;
    if (blockIdx.x < A) {
        lo = bounds[blockIdx.x];
        hi = bounds[blockIdx.x + 1];
#pragma unroll
        for (uint32_t k = 0; k < kSaltPre; ++k)
            pre[k] = load_word((lo >> 5) + k * kSaltThreads + tid, lo, hi);
    }
    if (blockIdx.x + G < A) {
        lo2 = bounds[blockIdx.x + G];
        hi2 = bounds[blockIdx.x + G + 1];
    }
    for (uint32_t a = blockIdx.x; a < A; a += G) {
        const uint32_t w_lo = lo >> 5, w_hi = lo < hi ? (hi - 1) >> 5 : 0;
        const uint32_t cur_lo = lo, cur_hi = hi;
        uint32_t cur[kSaltPre];
#pragma unroll
        for (uint32_t k = 0; k < kSaltPre; ++k) cur[k] = pre[k];
        lo = lo2;
        hi = hi2;
        if (a + G < A) {
#pragma unroll
            for (uint32_t k = 0; k < kSaltPre; ++k)
                pre[k] = load_word((lo >> 5) + k * kSaltThreads + tid, lo, hi);
        }
        if (a + 2 * G < A) {
            lo2 = bounds[a + 2 * G];
            hi2 = bounds[a + 2 * G + 1];
        }
        uint32_t salt = 0;
        if (cur_lo < cur_hi) {
            for (salt = 0; salt < kSaltLimit; ++salt) {
                const uint32_t sw0 = seed_word(seed, 3 * salt), sw1 = seed_word(seed, 3 * salt + 1),
                               sw2 = seed_word(seed, 3 * salt + 2);
                for (uint32_t c = tid; c < m_sub; c += kSaltThreads) head[c] = kNoLink;
                if (tid == 0) s_n = s_dup = 0;
                __syncthreads();
                uint32_t k = 0;
                for (uint32_t base = w_lo + (tid - lane); base <= w_hi; base += kSaltThreads, ++k) {
                    // (wave-uniform loop: the numbering below is a wave-wide scan)
                    uint32_t word = k < kSaltPre ? cur[k < kSaltPre ? k : 0]
                                                 : load_word(base + lane, cur_lo, cur_hi);
                    const uint32_t pc = __popc(word);
                    const uint32_t inc = wave_incl_scan<uint32_t>(pc);
                    const uint32_t tot = __builtin_amdgcn_readlane(inc, 63);
                    if (tot == 0) continue;
                    uint32_t start = 0;
                    if (lane == 0) start = atomicAdd(&s_n, tot);
                    start = __builtin_amdgcn_readfirstlane(start);
                    uint32_t t = start + inc - pc;
                    for (; word; word &= word - 1, ++t)  // (a partition holds <= P_cap)
                        if (t < P_cap) tag[t] = (base + lane) * 32 + uint32_t(__builtin_ctz(word));
                }
                __syncthreads();
                // every lane busy: the numbered non-zeros are hashed in number order (a
                // lane's own Index word holds anything from none to a dozen of them)
                for (uint32_t t = tid; t < min(s_n, P_cap); t += kSaltThreads) {
                    const uint32_t i = tag[t];
                    uint32_t neg;
                    const uint32_t c0 = hash_slot(i, sw0, m_sub, &neg);
                    tag[t] = hash_slot(i, sw1, m_sub, &neg) | (hash_slot(i, sw2, m_sub, &neg) << 16);
                    link[t] = uint16_t(atomicExch(&head[c0], t));
                }
                __syncthreads();
                const uint32_t n = min(s_n, P_cap);
                bool dup = false;
                for (uint32_t t = tid; t < n; t += kSaltThreads) {
                    const uint32_t mine = tag[t];
                    for (uint32_t p = link[t]; p != kNoLink; p = link[p]) dup |= tag[p] == mine;
                }
                if (dup) s_dup = 1;
                __syncthreads();
                const bool again = s_dup != 0;
                __syncthreads();  // s_dup is cleared by the next try
                if (!again) break;
            }
            salt = min(salt, kSaltLimit - 1);
        }
        if (tid == 0) salt_out[a] = salt;
    }
}

}  // namespace

size_t salt_lds_bytes(uint32_t T_cap, uint32_t P_cap)
{
    return size_t(P_cap) * 4 + size_t(T_cap / 3) * 4 + size_t(P_cap) * 2 + 16;
}

int launch_index_or(const tagc_plan_t *p, const tagc_rank_buffers *ranks, uint32_t n_ranks,
                    const tagc_shared_buffers *sh, hipStream_t s)
{
    const uint32_t n_words = uint32_t(p->n_c / 32);
    const uint32_t n_chunks = uint32_t(p->n_chunks);
    uint32_t *chunk = static_cast<uint32_t *>(sh->workspace);
    if (n_chunks) {
        ProfileScope ps("index_or", s);
        for (uint32_t r0 = 0; r0 < n_ranks; r0 += kMaxRanksPerPass) {
            RankPtrs rp{};
            const uint32_t n_in = std::min(kMaxRanksPerPass, n_ranks - r0);
            for (uint32_t r = 0; r < n_in; ++r) rp.p[r] = ranks[r0 + r].bitmap;
            const bool last = r0 + n_in == n_ranks;
            // the 4-bit running sum lives behind the chunk prefixes (the plan sized it)
            uint32_t *sum4 = chunk + ((size_t(n_chunks) + 1 + 3) & ~size_t(3));
            auto kernel = p->cfg.index_mode == TAGC_INDEX_ADD4
                              ? index_merge_kernel<TAGC_INDEX_ADD4>
                              : (p->cfg.index_mode == TAGC_INDEX_ADD1
                                     ? index_merge_kernel<TAGC_INDEX_ADD1>
                                     : index_merge_kernel<TAGC_INDEX_OR1>);
            kernel<<<n_chunks, 256, 0, s>>>(rp, n_in, sh->bitmap, n_words, r0 != 0, last, sum4,
                                            last ? chunk : nullptr);
        }
    }
    {
        ProfileScope ps("header", s);
        LayoutParams lp{p->cfg.sizing, p->cfg.sizing_milli, p->P_cap, p->T_cap,
                        p->n_real,     p->U_cap,            p->A_cap, p->m_cap};
        header_kernel<<<1, 1024, 0, s>>>(chunk, n_chunks, lp, sh->header, sh->status);
    }
    if (n_chunks) {
        ProfileScope ps("bounds", s);
        const uint32_t grid = uint32_t((p->A_cap + 1 + 3) / 4);
        bounds_kernel<<<grid, 256, 0, s>>>(sh->bitmap, n_words, uint32_t(p->n_c), chunk, n_chunks,
                                           sh->header, sh->bounds);
    }
    if (n_chunks) {
        ProfileScope ps("salt", s);
        const size_t lds = salt_lds_bytes(p->T_cap, p->P_cap);
        static size_t attr_bytes = 0;
        if (lds > attr_bytes) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(salt_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(lds)) != hipSuccess)
                return TAGC_EHIP;
            attr_bytes = lds;
        }
        // as many workgroups as fit the device at once, each taking partitions b, b + grid, ...
        const uint32_t per_cu = uint32_t(std::max<size_t>(1, std::min<size_t>(2, kLdsBytes / (lds + 1024))));
        const uint32_t grid = uint32_t(std::min<uint64_t>(p->A_cap, uint64_t(device_cu_count()) * per_cu));
        salt_kernel<<<grid, kSaltThreads, lds, s>>>(sh->bitmap, n_words, sh->header, sh->bounds,
                                                    sh->bounds + p->A_cap + 1, p->cfg.seed,
                                                    p->P_cap, p->T_cap / 3);
    }
    if (n_chunks) {
        ProfileScope ps("ranges", s);
        for (uint32_t r0 = 0; r0 < n_ranks; r0 += kMaxRanksPerPass) {
            RankPtrs ri{}, rc{};
            const uint32_t n_in = std::min(kMaxRanksPerPass, n_ranks - r0);
            for (uint32_t r = 0; r < n_in; ++r) {
                ri.p[r] = ranks[r0 + r].idx;
                rc.p[r] = ranks[r0 + r].cnt;
            }
            const uint64_t threads = uint64_t(n_in) * (p->A_cap + 1);
            ranges_kernel<<<uint32_t((threads + 255) / 256), 256, 0, s>>>(
                ri, rc, n_in, sh->header, sh->bounds, uint32_t(p->A_cap), p->cnt_ranges,
                uint32_t(p->K));
        }
    }
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
