// Count Sketch encode and aggregation.
//
// encode: local_count_sketch <- compress(g_shard, index) of Algorithm 1.  The merged Index
//   enters through the layout (and, when it was merged by addition, as a mask): partition a owns the pairs whose c-index lies in
//   [bounds[a], bounds[a+1]) -- a contiguous run of the rank's sorted pair list, whose ends
//   the Index aggregation leaves in the rank's cnt buffer -- and the
//   3*m_sub cells starting at a*3*m_sub.  One workgroup builds one sub-table (partition a,
//   hash function j) in LDS and writes it out once, so the sketch is produced with
//   coalesced stores and no global atomics.
// sum: Reduce(local_count_sketch, d) as an element-wise float32 sum in rank order.
#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

__global__ void __launch_bounds__(256)
encode_kernel(const uint32_t *__restrict__ idx, const float *__restrict__ val,
              const uint32_t *__restrict__ cnt, const uint32_t *__restrict__ header,
              float *__restrict__ sketch, uint32_t sw0, uint32_t sw1, uint32_t sw2,
              uint32_t ranges_off, uint32_t pair_cap, const uint32_t *__restrict__ mask)
{
    extern __shared__ float tile[];
    const uint32_t A = header[TAGC_HDR_A], m_sub = header[TAGC_HDR_MSUB];
    const uint32_t a = blockIdx.x, j = blockIdx.y;
    if (a >= A) return;
    const uint32_t sw = j == 0 ? sw0 : (j == 1 ? sw1 : sw2);
    // the partition's run of the sorted pair list, found when the Index was aggregated
    const uint32_t lo = min(cnt[ranges_off + a], pair_cap);
    const uint32_t hi = min(cnt[ranges_off + a + 1], pair_cap);
    // a thread's first pairs (all of them for a partition of up to 1024 pairs of this rank)
    // are requested together, before the tile is cleared
    // after an addition-simulated Index All-Reduce (section 2.2) the merged Index need not
    // hold every pair: only the positions it names are encoded (mask = merged Index then)
    auto named = [&](uint32_t i) { return !mask || ((mask[i >> 5] >> (i & 31)) & 1u); };
    constexpr uint32_t PRE = 4;
    uint32_t pi[PRE];
    float pv[PRE];
#pragma unroll
    for (uint32_t u = 0; u < PRE; ++u) {
        const uint32_t t = lo + threadIdx.x + u * 256;
        pi[u] = t < hi ? idx[t] : 0u;
        pv[u] = t < hi ? val[t] : 0.0f;
    }
    for (uint32_t c = threadIdx.x; c < m_sub; c += 256) tile[c] = 0.0f;
    __syncthreads();
#pragma unroll
    for (uint32_t u = 0; u < PRE; ++u) {
        if (lo + threadIdx.x + u * 256 < hi && named(pi[u])) {
            uint32_t neg;
            const uint32_t slot = hash_slot(pi[u], sw, m_sub, &neg);
            lds_add_f32(&tile[slot], neg ? -pv[u] : pv[u]);
        }
    }
    for (uint32_t t = lo + threadIdx.x + PRE * 256; t < hi; t += 256) {
        const uint32_t i = idx[t];
        const float v = val[t];
        if (!named(i)) continue;
        uint32_t neg;
        const uint32_t slot = hash_slot(i, sw, m_sub, &neg);
        lds_add_f32(&tile[slot], neg ? -v : v);
    }
    __syncthreads();
    // the tile leaves in 16-byte stores where the sketch is aligned for them
    const uint64_t b0 = (uint64_t(a) * 3 + j) * m_sub;
    float *out = sketch + b0;
    const uint32_t head = min(m_sub, uint32_t((4u - uint32_t(b0 & 3u)) & 3u));
    const uint32_t n4 = (m_sub - head) / 4;
    if (threadIdx.x < head) out[threadIdx.x] = tile[threadIdx.x];
    for (uint32_t v = threadIdx.x; v < n4; v += 256) {
        const float *t = tile + head + 4 * v;
        *reinterpret_cast<float4 *>(out + head + 4 * v) = make_float4(t[0], t[1], t[2], t[3]);
    }
    for (uint32_t c = head + 4 * n4 + threadIdx.x; c < m_sub; c += 256) out[c] = tile[c];
}

// Each workgroup sums tiles of kSumRows x 256 float4 cells: per rank it reads one
// contiguous 16 KiB piece (four loads per thread in flight), ranks in order.
constexpr uint32_t kSumRows = 4;

__global__ void __launch_bounds__(256)
sketch_sum_kernel(RankPtrs rp, uint32_t n_in, float *__restrict__ out,
                  const uint32_t *__restrict__ header, int accumulate)
{
    const uint32_t m = header[TAGC_HDR_M];
    const uint32_t m4 = m / 4;
    constexpr uint32_t TILE = 256 * kSumRows;
    for (uint32_t c0 = blockIdx.x * TILE; c0 < m4; c0 += gridDim.x * TILE) {
        float4 acc[kSumRows];
        const uint32_t c = c0 + threadIdx.x;
        uint32_t r = 0;
        const float4 *first = accumulate ? reinterpret_cast<const float4 *>(out)
                                         : static_cast<const float4 *>(rp.p[0]);
        if (!accumulate) r = 1;
#pragma unroll
        for (uint32_t i = 0; i < kSumRows; ++i)
            acc[i] = c + i * 256 < m4 ? first[c + i * 256] : make_float4(0.f, 0.f, 0.f, 0.f);
        for (; r < n_in; ++r) {
            const float4 *src = static_cast<const float4 *>(rp.p[r]);
            float4 v[kSumRows];
#pragma unroll
            for (uint32_t i = 0; i < kSumRows; ++i)
                v[i] = c + i * 256 < m4 ? src[c + i * 256] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (uint32_t i = 0; i < kSumRows; ++i) {
                acc[i].x += v[i].x; acc[i].y += v[i].y; acc[i].z += v[i].z; acc[i].w += v[i].w;
            }
        }
#pragma unroll
        for (uint32_t i = 0; i < kSumRows; ++i)
            if (c + i * 256 < m4) reinterpret_cast<float4 *>(out)[c + i * 256] = acc[i];
    }
    if (blockIdx.x == 0) {
        const uint32_t c = m4 * 4 + threadIdx.x;
        if (c < m) {
            float acc;
            uint32_t r = 0;
            if (accumulate) {
                acc = out[c];
            } else {
                acc = static_cast<const float *>(rp.p[0])[c];
                r = 1;
            }
            for (; r < n_in; ++r) acc += static_cast<const float *>(rp.p[r])[c];
            out[c] = acc;
        }
    }
}

}  // namespace

int launch_encode(const tagc_plan_t *p, const tagc_rank_buffers *rk, const tagc_shared_buffers *sh,
                  hipStream_t s)
{
    ProfileScope ps("encode", s);
    const size_t lds = size_t(p->T_cap / 3) * sizeof(float);
    dim3 grid(uint32_t(p->A_cap), 3, 1);
    encode_kernel<<<grid, 256, lds, s>>>(rk->idx, rk->val, rk->cnt, sh->header, rk->sketch,
                                         p->seed_word[0], p->seed_word[1], p->seed_word[2],
                                         p->cnt_ranges, uint32_t(p->K),
                                         p->cfg.index_mode == TAGC_INDEX_OR1 ? nullptr : sh->bitmap);
    return hip_ok(hipGetLastError());
}

int launch_sketch_sum(const tagc_plan_t *p, const tagc_rank_buffers *ranks, uint32_t n_ranks,
                      const tagc_shared_buffers *sh, hipStream_t s)
{
    ProfileScope ps("sketch_sum", s);
    const uint64_t m4cap = p->m_cap / 4 + 1;
    const uint64_t tile = 256 * kSumRows;
    const uint32_t grid = uint32_t(std::max<uint64_t>(
        1, std::min<uint64_t>((m4cap + tile - 1) / tile, uint64_t(device_cu_count()) * 8)));
    for (uint32_t r0 = 0; r0 < n_ranks; r0 += kMaxRanksPerPass) {
        RankPtrs rp{};
        const uint32_t n_in = std::min(kMaxRanksPerPass, n_ranks - r0);
        for (uint32_t r = 0; r < n_in; ++r) rp.p[r] = ranks[r0 + r].sketch;
        sketch_sum_kernel<<<grid, 256, 0, s>>>(rp, n_in, sh->sketch, sh->header, r0 != 0);
    }
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
