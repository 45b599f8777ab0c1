// Count Sketch encode and aggregation.
//
// encode: local_count_sketch <- compress(g_shard, index) of Algorithm 1.  The merged Index
//   enters through the layout only: partition a owns the pairs whose c-index lies in
//   [bounds[a], bounds[a+1]) -- a contiguous run of the rank's sorted pair list -- and the
//   3*m_sub cells starting at a*3*m_sub.  One workgroup builds one sub-table (partition a,
//   hash function j) in LDS and writes it out once, so the sketch is produced with
//   coalesced stores and no global atomics.
// sum: Reduce(local_count_sketch, d) as an element-wise float32 sum in rank order.
#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

// lower_bound over a sorted array by one wave: every step probes 64 evenly spaced
// positions at once, so a list of millions of pairs needs 4 dependent loads, not 21.
__device__ inline uint32_t wave_lower_bound(const uint32_t *__restrict__ a, uint32_t n,
                                            uint32_t key)
{
    const uint32_t lane = lane_id();
    uint32_t lo = 0, hi = n;  // answer in [lo, hi]; a[lo-1] < key <= a[hi]
    while (hi - lo > 64) {
        const uint32_t step = (hi - lo + 64) / 65;       // 64 probes split the range in 65
        const uint32_t pos = lo + (lane + 1) * step - 1;  // probe positions, ascending
        const bool lt = pos < hi && a[min(pos, n - 1)] < key;
        const uint32_t n_lt = __popcll(__ballot(lt));     // probes below the key (a prefix)
        const uint32_t new_lo = lo + n_lt * step;
        const uint32_t new_hi = n_lt == 64 ? hi : min(hi, lo + (n_lt + 1) * step - 1);
        lo = min(new_lo, hi);
        hi = new_hi;
    }
    const uint32_t pos = lo + lane;
    const bool lt = pos < hi && a[pos] < key;
    return lo + __popcll(__ballot(lt));
}

__global__ void __launch_bounds__(256)
encode_kernel(const uint32_t *__restrict__ idx, const float *__restrict__ val,
              const uint32_t *__restrict__ cnt, const uint32_t *__restrict__ header,
              const uint32_t *__restrict__ bounds, float *__restrict__ sketch, uint32_t sw0,
              uint32_t sw1, uint32_t sw2, uint32_t pair_cap)
{
    extern __shared__ float tile[];
    __shared__ uint32_t s_range[2];
    const uint32_t A = header[TAGC_HDR_A], m_sub = header[TAGC_HDR_MSUB];
    const uint32_t a = blockIdx.x, j = blockIdx.y;
    if (a >= A) return;
    const uint32_t sw = j == 0 ? sw0 : (j == 1 ? sw1 : sw2);
    for (uint32_t c = threadIdx.x; c < m_sub; c += 256) tile[c] = 0.0f;
    if (threadIdx.x < 128) {  // waves 0 and 1 search one bound each
        const uint32_t n = min(cnt[TAGC_CNT_TOTAL], pair_cap);
        const uint32_t w = threadIdx.x >> 6;
        const uint32_t r = wave_lower_bound(idx, n, bounds[a + w]);
        if ((threadIdx.x & 63) == 0) s_range[w] = r;
    }
    __syncthreads();
    const uint32_t lo = s_range[0], hi = s_range[1];
    for (uint32_t t = lo + threadIdx.x; t < hi; t += 256) {
        const uint32_t i = idx[t];
        const float v = val[t];
        uint32_t neg;
        const uint32_t slot = hash_slot(i, sw, m_sub, &neg);
        lds_add_f32(&tile[slot], neg ? -v : v);
    }
    __syncthreads();
    float *out = sketch + (uint64_t(a) * 3 + j) * m_sub;
    for (uint32_t c = threadIdx.x; c < m_sub; c += 256) out[c] = tile[c];
}

__global__ void __launch_bounds__(256)
sketch_sum_kernel(RankPtrs rp, uint32_t n_in, float *__restrict__ out,
                  const uint32_t *__restrict__ header, int accumulate)
{
    const uint32_t m = header[TAGC_HDR_M];
    const uint32_t m4 = m / 4;
    for (uint32_t c = blockIdx.x * 256 + threadIdx.x; c < m4; c += gridDim.x * 256) {
        float4 acc;
        uint32_t r = 0;
        if (accumulate) {
            acc = reinterpret_cast<const float4 *>(out)[c];
        } else {
            acc = static_cast<const float4 *>(rp.p[0])[c];
            r = 1;
        }
        for (; r < n_in; ++r) {
            float4 v = static_cast<const float4 *>(rp.p[r])[c];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        reinterpret_cast<float4 *>(out)[c] = acc;
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
    encode_kernel<<<grid, 256, lds, s>>>(rk->idx, rk->val, rk->cnt, sh->header, sh->bounds,
                                         rk->sketch, p->seed_word[0], p->seed_word[1],
                                         p->seed_word[2], uint32_t(p->K));
    return hip_ok(hipGetLastError());
}

int launch_sketch_sum(const tagc_plan_t *p, const tagc_rank_buffers *ranks, uint32_t n_ranks,
                      const tagc_shared_buffers *sh, hipStream_t s)
{
    ProfileScope ps("sketch_sum", s);
    const uint64_t m4cap = p->m_cap / 4 + 1;
    const uint32_t grid = uint32_t(
        std::max<uint64_t>(1, std::min<uint64_t>((m4cap + 255) / 256, uint64_t(device_cu_count()) * 16)));
    for (uint32_t r0 = 0; r0 < n_ranks; r0 += kMaxRanksPerPass) {
        RankPtrs rp{};
        const uint32_t n_in = std::min(kMaxRanksPerPass, n_ranks - r0);
        for (uint32_t r = 0; r < n_in; ++r) rp.p[r] = ranks[r0 + r].sketch;
        sketch_sum_kernel<<<grid, 256, 0, s>>>(rp, n_in, sh->sketch, sh->header, r0 != 0);
    }
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
