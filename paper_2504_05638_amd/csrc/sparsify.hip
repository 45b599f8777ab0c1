// Stage 1 of the hot path: dynamic magnitude sparsifier + local Index.
//
// For every compressed segment of one rank's gradient bucket: find the threshold key T
// such that exactly k_l entries survive (section 3.2: the zeroing value is chosen
// dynamically so that at least theta of the values become zero), then emit the
// survivors as (c-index, float32 value) pairs in ascending c-index together with the
// 1-bit-per-parameter Index (Algorithm 1: sparsify, create_index).
//
// Kernels
//   fill_zero      clears the per-call part of the workspace
//   hist1          exact histogram of the top 15 key bits (all of a bf16 key) in LDS
//   select1        threshold bin from that histogram
//   hist2/select2  fp32 only: the low 16 key bits inside the threshold bin
//   compact        one ordered pass: survivors + Index words, decoupled look-back
//
// Keys: |g| as an unsigned integer (bit pattern with the sign cleared).  Ties at the
// threshold are broken towards the lower position; exact zeros never survive.
#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

constexpr int kF32 = TAGC_F32, kBF16 = TAGC_BF16;

__global__ void __launch_bounds__(256) fill_zero_kernel(uint4 *p, uint64_t n16, uint32_t *cnt,
                                                        uint32_t n_cnt)
{
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (uint64_t i = blockIdx.x * 256ull + threadIdx.x; i < n16; i += gridDim.x * 256ull)
        p[i] = z;
    if (blockIdx.x == 0)
        for (uint32_t i = threadIdx.x; i < n_cnt; i += 256) cnt[i] = 0;
}

// ------------------------------------------------------------------ hist1

template <int DTYPE>
__device__ inline void hist_word(uint32_t w, uint32_t *h)
{
    if (DTYPE == kBF16) {
        uint32_t a = w & 0x7FFFu, b = (w >> 16) & 0x7FFFu;
        if (a) atomicAdd(&h[a], 1u);
        if (b) atomicAdd(&h[b], 1u);
    } else {
        uint32_t key = w & 0x7FFFFFFFu;
        if (key) atomicAdd(&h[key >> 16], 1u);
    }
}

template <int DTYPE>
__device__ inline void hist_vec(uint4 v, uint32_t *h)
{
    hist_word<DTYPE>(v.x, h);
    hist_word<DTYPE>(v.y, h);
    hist_word<DTYPE>(v.z, h);
    hist_word<DTYPE>(v.w, h);
}

__device__ inline uint32_t load_elem_bits(const char *base, uint64_t i, int dtype)
{
    if (dtype == kBF16) return uint32_t(reinterpret_cast<const uint16_t *>(base)[i]) << 16;
    return reinterpret_cast<const uint32_t *>(base)[i];
}

template <int DTYPE>
__device__ inline void hist_elem(uint32_t f32bits, uint32_t *h)
{
    uint32_t key = f32bits & 0x7FFFFFFFu;
    if (key) atomicAdd(&h[key >> 16], 1u);
}

// One workgroup per CU, 32768 LDS counters.  Segments are processed one after another;
// after each the non-zero counters are added to the segment's global histogram.
template <int DTYPE>
__global__ void __launch_bounds__(kHistThreads)
hist1_kernel(const char *__restrict__ grad, const uint32_t *__restrict__ table,
             uint32_t *__restrict__ hist)
{
    extern __shared__ uint32_t h[];
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < kBins1; i += kHistThreads) h[i] = 0;
    __syncthreads();
    for (uint32_t l = 0; l < L; ++l) {
        const SegDev sd = segs[l];
        if (sd.k == 0 || sd.n == 0) continue;
        const char *base = grad + sd.offset * EB;
        if (sd.aligned) {
            const uint4 *vp = reinterpret_cast<const uint4 *>(base);
            const uint64_t nvec = sd.n / VEC;
            const uint64_t stride = uint64_t(gridDim.x) * kHistThreads;
            uint64_t v = uint64_t(blockIdx.x) * kHistThreads + tid;
            for (; v + 3 * stride < nvec; v += 4 * stride) {
                uint4 a = vp[v], b = vp[v + stride], c = vp[v + 2 * stride],
                      d = vp[v + 3 * stride];
                hist_vec<DTYPE>(a, h);
                hist_vec<DTYPE>(b, h);
                hist_vec<DTYPE>(c, h);
                hist_vec<DTYPE>(d, h);
            }
            for (; v < nvec; v += stride) hist_vec<DTYPE>(vp[v], h);
            if (blockIdx.x == 0) {
                uint64_t i = nvec * VEC + tid;
                if (i < sd.n) hist_elem<DTYPE>(load_elem_bits(base, i, DTYPE), h);
            }
        } else {
            for (uint64_t i = uint64_t(blockIdx.x) * kHistThreads + tid; i < sd.n;
                 i += uint64_t(gridDim.x) * kHistThreads)
                hist_elem<DTYPE>(load_elem_bits(base, i, DTYPE), h);
        }
        __syncthreads();
        uint32_t *gh = hist + uint64_t(l) * kBins1;
        for (uint32_t i = tid; i < kBins1; i += kHistThreads) {
            uint32_t c = h[i];
            if (c) {
                atomicAdd(&gh[i], c);
                h[i] = 0;
            }
        }
        __syncthreads();
    }
}

// ----------------------------------------------------------------- select

// Largest bin b with  sum_{x >= b} hist[x] >= need  (need >= 1).  1024 threads, thread t
// owns the BPT consecutive bins starting at t*BPT.  Returns false if the whole histogram
// holds fewer than `need`; *total_out is the histogram's sum either way.
template <int BPT>
__device__ inline bool select_bins(const uint32_t *__restrict__ hist, uint32_t need,
                                   uint32_t *bin_out, uint32_t *above_out, uint32_t *at_out,
                                   uint32_t *total_out, uint32_t *smem /* >= 20 words */)
{
    const uint32_t t = threadIdx.x;
    const uint4 *hv = reinterpret_cast<const uint4 *>(hist + uint64_t(t) * BPT);
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < BPT / 4; ++i) {
        uint4 v = hv[i];
        s += v.x + v.y + v.z + v.w;
    }
    uint32_t total;
    uint32_t prefix = block_excl_scan<uint32_t, kHistThreads / 64>(s, &total, smem);
    uint32_t suffix = total - prefix;  // bins of this thread and all higher ones
    if (total >= need && suffix >= need && suffix - s < need) {
        uint32_t acc = suffix - s;
        for (int b = BPT - 1; b >= 0; --b) {
            uint32_t c = hist[uint64_t(t) * BPT + b];
            if (acc + c >= need) {
                smem[16] = t * BPT + b;
                smem[17] = acc;
                smem[18] = c;
                break;
            }
            acc += c;
        }
    }
    __syncthreads();
    *bin_out = smem[16];
    *above_out = smem[17];
    *at_out = smem[18];
    *total_out = total;
    __syncthreads();
    return total >= need;
}

template <int DTYPE>
__global__ void __launch_bounds__(kHistThreads)
select1_kernel(const uint32_t *__restrict__ table, const uint32_t *__restrict__ hist,
               SelDev *__restrict__ sel, uint32_t *__restrict__ cnt)
{
    __shared__ uint32_t smem[32];
    const uint32_t l = blockIdx.x;
    const SegDev sd = reinterpret_cast<const SegDev *>(table + 8)[l];
    SelDev r{};
    if (sd.k == 0 || sd.n == 0) {
        r.T = 0xFFFFFFFFu;
        if (threadIdx.x == 0) {
            sel[l] = r;
            cnt[TAGC_CNT_SEG0 + l] = 0;
        }
        return;
    }
    const uint32_t *h = hist + uint64_t(l) * kBins1;
    // inputs with an all-ones exponent fall into bins >= 0x7F80
    {
        uint32_t nf = 0;
        if (threadIdx.x >= 0x7F80u / 32)
            for (int i = 0; i < 32; ++i) nf += h[threadIdx.x * 32 + i];
        nf = block_sum<uint32_t, kHistThreads / 64>(nf, smem);
        if (threadIdx.x == 0 && nf) atomicAdd(&cnt[TAGC_CNT_NONFINITE], nf);
    }
    uint32_t bin, above, at, total;
    bool found = select_bins<32>(h, sd.k, &bin, &above, &at, &total, smem);
    if (threadIdx.x != 0) return;
    if (!found) {  // fewer non-zeros than k: keep every non-zero
        r.T = 0;
        r.quota = 0;
        r.G = total;
        r.cnt = total;
    } else if (DTYPE == kBF16) {
        r.T = bin << 16;  // keys are compared as float32 bit patterns
        r.G = above;
        r.quota = sd.k - above;
        r.cnt = sd.k;
    } else {
        r.bin1 = bin;
        r.G1 = above;
        r.need2 = 1;
    }
    sel[l] = r;
    if (!r.need2) {
        cnt[TAGC_CNT_SEG0 + l] = r.cnt;
        atomicAdd(&cnt[TAGC_CNT_TOTAL], r.cnt);
    }
}

// fp32: histogram of the low 16 key bits of the entries inside the threshold bin.
__global__ void __launch_bounds__(256)
hist2_kernel(const char *__restrict__ grad, const uint32_t *__restrict__ table,
             const SelDev *__restrict__ sel, uint32_t *__restrict__ hist2)
{
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const uint32_t tid = threadIdx.x;
    for (uint32_t l = 0; l < L; ++l) {
        if (!sel[l].need2) continue;
        const SegDev sd = segs[l];
        const uint32_t bin1 = sel[l].bin1;
        uint32_t *gh = hist2 + uint64_t(l) * kBins2;
        const char *base = grad + sd.offset * 4;
        if (sd.aligned) {
            const uint4 *vp = reinterpret_cast<const uint4 *>(base);
            const uint64_t nvec = sd.n / 4;
            for (uint64_t v = blockIdx.x * 256ull + tid; v < nvec; v += gridDim.x * 256ull) {
                uint4 q = vp[v];
                uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t key = w[e] & 0x7FFFFFFFu;
                    if (key && (key >> 16) == bin1) atomicAdd(&gh[key & 0xFFFFu], 1u);
                }
            }
            if (blockIdx.x == 0) {
                uint64_t i = nvec * 4 + tid;
                if (i < sd.n) {
                    uint32_t key = reinterpret_cast<const uint32_t *>(base)[i] & 0x7FFFFFFFu;
                    if (key && (key >> 16) == bin1) atomicAdd(&gh[key & 0xFFFFu], 1u);
                }
            }
        } else {
            for (uint64_t i = blockIdx.x * 256ull + tid; i < sd.n; i += gridDim.x * 256ull) {
                uint32_t key = reinterpret_cast<const uint32_t *>(base)[i] & 0x7FFFFFFFu;
                if (key && (key >> 16) == bin1) atomicAdd(&gh[key & 0xFFFFu], 1u);
            }
        }
    }
}

__global__ void __launch_bounds__(kHistThreads)
select2_kernel(const uint32_t *__restrict__ table, const uint32_t *__restrict__ hist2,
               SelDev *__restrict__ sel, uint32_t *__restrict__ cnt)
{
    __shared__ uint32_t smem[32];
    const uint32_t l = blockIdx.x;
    SelDev r = sel[l];
    if (!r.need2) return;
    const SegDev sd = reinterpret_cast<const SegDev *>(table + 8)[l];
    uint32_t bin, above, at, total;
    bool found =
        select_bins<64>(hist2 + uint64_t(l) * kBins2, sd.k - r.G1, &bin, &above, &at, &total, smem);
    if (threadIdx.x != 0) return;
    if (!found) {  // cannot happen when hist1 and hist2 saw the same data
        bin = 0;
        above = total;
        atomicOr(&cnt[TAGC_CNT_FLAGS], TAGC_FLAG_OVERFLOW);
    }
    r.T = (r.bin1 << 16) | bin;
    r.G = r.G1 + above;
    r.quota = sd.k - r.G;
    r.cnt = sd.k;
    r.need2 = 0;
    sel[l] = r;
    cnt[TAGC_CNT_SEG0 + l] = r.cnt;
    atomicAdd(&cnt[TAGC_CNT_TOTAL], r.cnt);
}

// ---------------------------------------------------------------- compact

constexpr uint64_t kStAgg = 1ull << 62, kStPre = 2ull << 62, kStMask = 3ull << 62;

// Decoupled look-back over the tiles of one segment, run by the first wave of the
// workgroup.  state word = status(2) | count(key > T)(31) | count(key == T)(31).
// The grid is persistent and fully resident, and workgroup b takes tiles b, b+G, b+2G, ...;
// so every predecessor tile this waits for belongs to a workgroup that is running and
// that publishes its counts without waiting for any later tile.
__device__ inline uint64_t lookback(uint64_t *state, uint32_t t, uint32_t t0, uint64_t agg,
                                    uint32_t *flags)
{
    const uint32_t l = lane_id();
    if (t == t0) {
        if (l == 0) st_agent(&state[t], kStPre | agg);
        return 0;
    }
    if (l == 0) st_agent(&state[t], kStAgg | agg);
    uint64_t excl = 0;
    int64_t j = int64_t(t) - 1;
    uint32_t spins = 0;
    while (true) {
        const int64_t i = j - l;
        const bool real = i >= int64_t(t0);
        uint64_t s = real ? ld_agent(&state[i]) : kStPre;
        while (__any((s & kStMask) == 0)) {
            if (++spins > kSpinLimit) {
                if (l == 0) atomicOr(flags, TAGC_FLAG_SPIN_LIMIT);
                s |= kStPre;  // give up: result invalid, but every wave still exits
                break;
            }
            __builtin_amdgcn_s_sleep(1);
            if ((s & kStMask) == 0) s = ld_agent(&state[i]);
        }
        const uint64_t pm = __ballot((s & kStMask) == kStPre);
        const uint64_t v = s & ~kStMask;
        if (pm) {
            const uint32_t first = __builtin_ctzll(pm);
            excl += wave_sum<uint64_t>(l <= first ? v : 0ull);
            break;
        }
        excl += wave_sum<uint64_t>(v);
        j -= 64;
    }
    if (l == 0) st_agent(&state[t], kStPre | (excl + agg));
    return excl;
}

template <int DTYPE>
__global__ void __launch_bounds__(kCompactThreads)
compact_kernel(const char *__restrict__ grad, const uint32_t *__restrict__ table,
               const SelDev *__restrict__ sel, uint64_t *tile_state, uint32_t *ticket,
               uint32_t *__restrict__ idx_out, float *__restrict__ val_out,
               uint32_t *__restrict__ bitmap, uint32_t *cnt)
{
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    constexpr uint32_t ROWS = kCompactRows;
    constexpr uint32_t ROW_ELEMS = kCompactThreads * VEC;
    constexpr uint32_t TILE = ROW_ELEMS * ROWS;
    constexpr uint32_t LPW = 32 / VEC;  // lanes that share one Index word
    __shared__ uint64_t s_scan[2 * (kCompactThreads / 64)];
    __shared__ uint64_t s_excl;
    __shared__ uint32_t s_base;

    const uint32_t L = table[0], total_tiles = table[1];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const uint32_t tid = threadIdx.x;

    for (uint32_t t = blockIdx.x; t < total_tiles; t += gridDim.x) {

        // segment of this tile: the last l with tile_start[l] <= t
        uint32_t lo = 0, hi = L;
        while (hi - lo > 1) {
            uint32_t mid = (lo + hi) >> 1;
            if (segs[mid].tile_start <= t) lo = mid; else hi = mid;
        }
        const uint32_t l = lo;
        const SegDev sd = segs[l];
        const SelDev se = sel[l];
        const uint32_t base_rel = (t - sd.tile_start) * TILE;
        const char *base = grad + sd.offset * EB;

        // ---- load (rows of 256 16-byte vectors, lane-contiguous)
        uint32_t w[ROWS][4];
        uint32_t gtm[ROWS], eqm[ROWS];
#pragma unroll
        for (uint32_t r = 0; r < ROWS; ++r) {
            w[r][0] = w[r][1] = w[r][2] = w[r][3] = 0;
            gtm[r] = eqm[r] = 0;
        }
        if (se.cnt != 0) {
#pragma unroll
            for (uint32_t r = 0; r < ROWS; ++r) {
                const uint32_t rel = base_rel + r * ROW_ELEMS + tid * VEC;
                if (rel >= sd.n) continue;
                if (sd.aligned && rel + VEC <= sd.n) {
                    uint4 q = *reinterpret_cast<const uint4 *>(base + uint64_t(rel) * EB);
                    w[r][0] = q.x; w[r][1] = q.y; w[r][2] = q.z; w[r][3] = q.w;
                } else {
                    const uint32_t cntv = min(VEC, sd.n - rel);
#pragma unroll
                    for (uint32_t e = 0; e < VEC; ++e) {
                        if (e >= cntv) continue;
                        if (DTYPE == kBF16) {
                            uint32_t b = reinterpret_cast<const uint16_t *>(base)[uint64_t(rel) + e];
                            w[r][e >> 1] |= b << (16 * (e & 1));
                        } else {
                            w[r][e] = reinterpret_cast<const uint32_t *>(base)[uint64_t(rel) + e];
                        }
                    }
                }
            }
            // ---- classify.  Elements past the end were loaded as 0 and are never kept.
#pragma unroll
            for (uint32_t r = 0; r < ROWS; ++r) {
#pragma unroll
                for (uint32_t e = 0; e < VEC; ++e) {
                    uint32_t bits = DTYPE == kBF16 ? ((w[r][e >> 1] >> (16 * (e & 1))) << 16)
                                                   : w[r][e];
                    uint32_t key = bits & 0x7FFFFFFFu;
                    if (key > se.T) gtm[r] |= 1u << e;
                    else if (key == se.T && se.quota) eqm[r] |= 1u << e;
                }
            }
        }
        uint64_t g = 0, q = 0;
#pragma unroll
        for (uint32_t r = 0; r < ROWS; ++r) {
            g |= uint64_t(__popc(gtm[r])) << (16 * r);
            q |= uint64_t(__popc(eqm[r])) << (16 * r);
        }
        // ---- workgroup scan of both packed counters (row totals stay below 2^16)
        uint64_t gtot, qtot;
        const uint64_t gex =
            block_excl_scan<uint64_t, kCompactThreads / 64>(g, &gtot, s_scan);
        const uint64_t qex =
            block_excl_scan<uint64_t, kCompactThreads / 64>(q, &qtot, s_scan);
        uint32_t Gr[ROWS], Er[ROWS], Gt = 0, Et = 0;
#pragma unroll
        for (uint32_t r = 0; r < ROWS; ++r) {
            Gr[r] = uint32_t(gtot >> (16 * r)) & 0xFFFFu;
            Er[r] = uint32_t(qtot >> (16 * r)) & 0xFFFFu;
            Gt += Gr[r];
            Et += Er[r];
        }
        // ---- look-back across the tiles of this segment + pair offset of the segment
        if (tid < 64) {
            uint64_t ex = lookback(tile_state, t, sd.tile_start, (uint64_t(Gt) << 31) | Et,
                                   &cnt[TAGC_CNT_FLAGS]);
            uint32_t sb = 0;
            for (uint32_t i = tid; i < l; i += 64) sb += sel[i].cnt;
            sb = wave_sum<uint32_t>(sb);
            if (tid == 0) {
                s_excl = ex;
                s_base = sb;
            }
        }
        __syncthreads();
        const uint64_t ex = s_excl;
        const uint32_t seg_base = s_base;
        uint32_t grun = uint32_t(ex >> 31), erun = uint32_t(ex & 0x7FFFFFFFu);

        // ---- emit pairs and Index words
        uint32_t keepm[ROWS];
#pragma unroll
        for (uint32_t r = 0; r < ROWS; ++r) {
            uint32_t gb = grun + (uint32_t(gex >> (16 * r)) & 0xFFFFu);
            uint32_t eb = erun + (uint32_t(qex >> (16 * r)) & 0xFFFFu);
            const uint32_t rel = base_rel + r * ROW_ELEMS + tid * VEC;
            uint32_t km = gtm[r];
            uint32_t m = gtm[r] | eqm[r];
            while (m) {
                const uint32_t e = __builtin_ctz(m);
                m &= m - 1;
                uint32_t pos;
                bool keep;
                if ((gtm[r] >> e) & 1u) {
                    pos = gb + min(eb, se.quota);
                    keep = true;
                    ++gb;
                } else {
                    pos = gb + eb;
                    keep = eb < se.quota;
                    ++eb;
                }
                if (keep) {
                    km |= 1u << e;
                    uint32_t bits = DTYPE == kBF16 ? ((w[r][e >> 1] >> (16 * (e & 1))) << 16)
                                                   : w[r][e];
                    idx_out[seg_base + pos] = sd.c_off + rel + e;
                    val_out[seg_base + pos] = __uint_as_float(bits);
                }
            }
            keepm[r] = km;
            grun += Gr[r];
            erun += Er[r];
        }
#pragma unroll
        for (uint32_t r = 0; r < ROWS; ++r) {
            const uint32_t rel = base_rel + r * ROW_ELEMS + tid * VEC;
            uint32_t v = keepm[r] << (VEC * (tid & (LPW - 1)));
#pragma unroll
            for (uint32_t d = 1; d < LPW; d <<= 1) v |= __shfl_xor(v, d, 64);
            const uint32_t rel0 = rel - (tid & (LPW - 1)) * VEC;  // first element of the word
            if ((tid & (LPW - 1)) == 0 && rel0 < sd.n) bitmap[(sd.c_off + rel0) >> 5] = v;
        }
        __syncthreads();  // s_excl / s_base are rewritten by the next iteration
    }
}

}  // namespace

// ------------------------------------------------------------------- host

int launch_sparsify(const tagc_plan_t *p, const void *grad, const tagc_rank_buffers *rk,
                    const tagc_shared_buffers *sh, hipStream_t s)
{
    const uint32_t L = uint32_t(p->table.size());
    const uint32_t *table = static_cast<const uint32_t *>(sh->table);
    char *ws = static_cast<char *>(rk->workspace);
    uint32_t *hist1 = reinterpret_cast<uint32_t *>(ws + p->ws.hist1);
    uint32_t *hist2 = reinterpret_cast<uint32_t *>(ws + p->ws.hist2);
    uint64_t *tile_state = reinterpret_cast<uint64_t *>(ws + p->ws.tile_state);
    uint32_t *counters = reinterpret_cast<uint32_t *>(ws + p->ws.counters);
    SelDev *sel = reinterpret_cast<SelDev *>(ws + p->ws.sel);
    const char *g = static_cast<const char *>(grad);
    const int cus = device_cu_count();
    const bool bf16 = p->cfg.dtype == TAGC_BF16;

    {
        ProfileScope ps("fill_zero", s);
        uint64_t n16 = p->zero_bytes / 16;
        uint32_t grid = uint32_t(std::min<uint64_t>((n16 + 255) / 256, uint64_t(cus) * 8));
        fill_zero_kernel<<<std::max(grid, 1u), 256, 0, s>>>(reinterpret_cast<uint4 *>(ws), n16,
                                                            rk->cnt, TAGC_CNT_SEG0 + L);
    }
    if (L == 0) return hip_ok(hipGetLastError());
    {
        ProfileScope ps("hist1", s);
        static bool attr_done[2] = {false, false};
        const size_t lds = kBins1 * sizeof(uint32_t);
        if (bf16) {
            if (!attr_done[1]) {
                if (hipFuncSetAttribute(reinterpret_cast<const void *>(hist1_kernel<kBF16>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                        int(lds)) != hipSuccess)
                    return TAGC_EHIP;
                attr_done[1] = true;
            }
            hist1_kernel<kBF16><<<cus, kHistThreads, lds, s>>>(g, table, hist1);
        } else {
            if (!attr_done[0]) {
                if (hipFuncSetAttribute(reinterpret_cast<const void *>(hist1_kernel<kF32>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                        int(lds)) != hipSuccess)
                    return TAGC_EHIP;
                attr_done[0] = true;
            }
            hist1_kernel<kF32><<<cus, kHistThreads, lds, s>>>(g, table, hist1);
        }
    }
    {
        ProfileScope ps("select1", s);
        if (bf16)
            select1_kernel<kBF16><<<L, kHistThreads, 0, s>>>(table, hist1, sel, rk->cnt);
        else
            select1_kernel<kF32><<<L, kHistThreads, 0, s>>>(table, hist1, sel, rk->cnt);
    }
    if (!bf16) {
        {
            ProfileScope ps("hist2", s);
            hist2_kernel<<<cus * 8, 256, 0, s>>>(g, table, sel, hist2);
        }
        {
            ProfileScope ps("select2", s);
            select2_kernel<<<L, kHistThreads, 0, s>>>(table, hist2, sel, rk->cnt);
        }
    }
    if (p->total_tiles) {
        ProfileScope ps("compact", s);
        // persistent grid that is resident as a whole (the look-back relies on it)
        static int per_cu[2] = {0, 0};
        int &occ = per_cu[bf16 ? 1 : 0];
        if (occ == 0) {
            int n = 0;
            hipError_t e = bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(
                                      &n, compact_kernel<kBF16>, kCompactThreads, 0)
                                : hipOccupancyMaxActiveBlocksPerMultiprocessor(
                                      &n, compact_kernel<kF32>, kCompactThreads, 0);
            if (e != hipSuccess || n <= 0) return TAGC_EHIP;
            occ = n;
        }
        uint32_t grid = std::min<uint32_t>(p->total_tiles, uint32_t(cus) * uint32_t(occ));
        if (bf16)
            compact_kernel<kBF16><<<grid, kCompactThreads, 0, s>>>(
                g, table, sel, tile_state, counters, rk->idx, rk->val, rk->bitmap, rk->cnt);
        else
            compact_kernel<kF32><<<grid, kCompactThreads, 0, s>>>(
                g, table, sel, tile_state, counters, rk->idx, rk->val, rk->bitmap, rk->cnt);
    }
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
