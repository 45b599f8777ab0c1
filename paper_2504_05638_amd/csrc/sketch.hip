// Count Sketch encode and aggregation.
//
// encode: local_count_sketch <- compress(g_shard, index) of Algorithm 1.  The merged Index
//   enters through the layout (and, when it was merged by addition, as a mask): partition a
//   owns the pairs whose c-index lies in [bounds[a], bounds[a+1]) -- a contiguous run of the
//   rank's sorted pair list, whose ends the Index aggregation leaves in the rank's cnt
//   buffer -- the 3*m_sub cells starting at a*3*m_sub, and its own salt for the hash functions
//   (also left by the Index aggregation, behind the bounds).  One workgroup builds the
//   partition's three sub-tables in LDS, reading the pairs once, and writes them out as one
//   contiguous run, so the sketch is produced with coalesced stores and no global atomics.
// sum: Reduce(local_count_sketch, d) as an element-wise float32 sum in rank order.
#include "device_utils.h"
#include "tagc_internal.h"

namespace tagc {

namespace {

constexpr uint32_t kEncodeThreads = 512;

__global__ void __launch_bounds__(kEncodeThreads)
encode_kernel(const uint32_t *__restrict__ idx, const float *__restrict__ val,
              const uint32_t *__restrict__ cnt, const uint32_t *__restrict__ header,
              float *__restrict__ sketch, uint64_t seed, const uint32_t *__restrict__ salt,
              uint32_t ranges_off, uint32_t pair_cap, const uint32_t *__restrict__ mask,
              uint32_t cells16)
{
    constexpr uint32_t NT = kEncodeThreads;
    extern __shared__ float tile[];  // the partition's three sub-tables, as in the sketch
    const uint32_t A = header[TAGC_HDR_A], m_sub = header[TAGC_HDR_MSUB];
    const uint32_t a = blockIdx.x;
    if (a >= A) return;
    const uint32_t cells = 3 * m_sub;
    // the partition's hash functions: the seed under the salt the Index aggregation chose
    const uint32_t sa = salt[a];
    const uint32_t sw0 = seed_word(seed, 3 * sa), sw1 = seed_word(seed, 3 * sa + 1),
                   sw2 = seed_word(seed, 3 * sa + 2);
    // the partition's run of the sorted pair list, found when the Index was aggregated
    const uint32_t lo = min(cnt[ranges_off + a], pair_cap);
    const uint32_t hi = min(cnt[ranges_off + a + 1], pair_cap);
    // after an addition-simulated Index All-Reduce (section 2.2) the merged Index need not
    // hold every pair: only the positions it names are encoded (mask = merged Index then)
    auto named = [&](uint32_t i) { return !mask || ((mask[i >> 5] >> (i & 31)) & 1u); };
    auto add = [&](uint32_t i, float v) {
        uint32_t neg;
        uint32_t slot = hash_slot(i, sw0, m_sub, &neg);
        lds_add_f32(&tile[slot], neg ? -v : v);
        slot = hash_slot(i, sw1, m_sub, &neg);
        lds_add_f32(&tile[m_sub + slot], neg ? -v : v);
        slot = hash_slot(i, sw2, m_sub, &neg);
        lds_add_f32(&tile[2 * m_sub + slot], neg ? -v : v);
    };
    // a thread's first pairs (all of them for a partition of up to 1024 pairs of this rank)
    // are requested together, before the tiles are cleared
    constexpr uint32_t PRE = 4;
    uint32_t pi[PRE];
    float pv[PRE];
#pragma unroll
    for (uint32_t u = 0; u < PRE; ++u) {
        const uint32_t t = lo + threadIdx.x + u * NT;
        pi[u] = t < hi ? idx[t] : 0u;
        pv[u] = t < hi ? val[t] : 0.0f;
    }
    for (uint32_t c = threadIdx.x; c < cells; c += NT) tile[c] = 0.0f;
    __syncthreads();
#pragma unroll
    for (uint32_t u = 0; u < PRE; ++u)
        if (lo + threadIdx.x + u * NT < hi && named(pi[u])) add(pi[u], pv[u]);
    for (uint32_t t = lo + threadIdx.x + PRE * NT; t < hi; t += NT) {
        const uint32_t i = idx[t];
        const float v = val[t];
        if (named(i)) add(i, v);
    }
    __syncthreads();
    // the partition's cells are one contiguous run of the sketch
    const uint64_t b0 = uint64_t(a) * cells;
    if (cells16) {
        // 16-bit cells on the wire: each cell rounded to the nearest bfloat16, ties to even;
        // eight to a 16-byte store where the sketch is aligned for them
        uint16_t *out = reinterpret_cast<uint16_t *>(sketch) + b0;
        const uint32_t head = min(cells, uint32_t((8u - uint32_t(b0 & 7u)) & 7u));
        const uint32_t n8 = (cells - head) / 8;
        if (threadIdx.x < head) out[threadIdx.x] = uint16_t(round_to_bf16(tile[threadIdx.x]));
        for (uint32_t v = threadIdx.x; v < n8; v += NT) {
            const float *t = tile + head + 8 * v;
            st_stream(reinterpret_cast<uint4 *>(out + head + 8 * v),
                      make_uint4(round_to_bf16(t[0]) | (round_to_bf16(t[1]) << 16),
                                 round_to_bf16(t[2]) | (round_to_bf16(t[3]) << 16),
                                 round_to_bf16(t[4]) | (round_to_bf16(t[5]) << 16),
                                 round_to_bf16(t[6]) | (round_to_bf16(t[7]) << 16)));
        }
        for (uint32_t c = head + 8 * n8 + threadIdx.x; c < cells; c += NT)
            out[c] = uint16_t(round_to_bf16(tile[c]));
        return;
    }
    // 16-byte stores where the sketch is aligned for them
    float *out = sketch + b0;
    const uint32_t head = min(cells, uint32_t((4u - uint32_t(b0 & 3u)) & 3u));
    const uint32_t n4 = (cells - head) / 4;
    if (threadIdx.x < head) out[threadIdx.x] = tile[threadIdx.x];
    for (uint32_t v = threadIdx.x; v < n4; v += NT) {
        const float *t = tile + head + 4 * v;
        st_stream(reinterpret_cast<float4 *>(out + head + 4 * v),
                  make_float4(t[0], t[1], t[2], t[3]));
    }
    for (uint32_t c = head + 4 * n4 + threadIdx.x; c < cells; c += NT) out[c] = tile[c];
}

// One float4 of cells per thread: the loads of up to kSumBatch ranks are issued together
// (streaming, each byte is read once) and added in rank order, ((C_0 + C_1) + C_2) + ...;
// more ranks than that take another round of loads, more than one launch holds continue
// from `out`.
constexpr uint32_t kSumBatch = 16;

__global__ void __launch_bounds__(256)
sketch_sum_kernel(RankPtrs rp, uint32_t n_in, float *__restrict__ out,
                  const uint32_t *__restrict__ header, int accumulate)
{
    const uint32_t m = header[TAGC_HDR_M];
    const uint32_t m4 = m / 4;
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;
    if (c < m4) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (accumulate) acc = reinterpret_cast<const float4 *>(out)[c];
        for (uint32_t r0 = 0; r0 < n_in; r0 += kSumBatch) {
            float4 v[kSumBatch];
#pragma unroll
            for (uint32_t i = 0; i < kSumBatch; ++i)
                if (r0 + i < n_in) v[i] = ld_stream(static_cast<const float4 *>(rp.p[r0 + i]) + c);
#pragma unroll
            for (uint32_t i = 0; i < kSumBatch; ++i) {
                if (r0 + i >= n_in) continue;
                if (r0 + i == 0 && !accumulate) {
                    acc = v[0];  // the first term as it is: -0 stays -0
                } else {
                    acc.x += v[i].x; acc.y += v[i].y; acc.z += v[i].z; acc.w += v[i].w;
                }
            }
        }
        st_stream(reinterpret_cast<float4 *>(out) + c, acc);
    }
    if (blockIdx.x == 0) {
        const uint32_t t = m4 * 4 + threadIdx.x;
        if (t < m) {
            float acc;
            uint32_t r = 0;
            if (accumulate) {
                acc = out[t];
            } else {
                acc = static_cast<const float *>(rp.p[0])[t];
                r = 1;
            }
            for (; r < n_in; ++r) acc += static_cast<const float *>(rp.p[r])[t];
            out[t] = acc;
        }
    }
}

// The same sum over ranks whose cells are bfloat16 on the wire: eight cells (one 16-byte
// load) per rank and thread, widened and added in float32 in rank order.
__global__ void __launch_bounds__(256)
sketch_sum16_kernel(RankPtrs rp, uint32_t n_in, float *__restrict__ out,
                    const uint32_t *__restrict__ header, int accumulate)
{
    const uint32_t m = header[TAGC_HDR_M];
    const uint32_t m8 = m / 8;
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;
    if (c < m8) {
        float acc[8];
        if (accumulate) {
            const float4 a = reinterpret_cast<const float4 *>(out)[2 * c];
            const float4 b = reinterpret_cast<const float4 *>(out)[2 * c + 1];
            acc[0] = a.x; acc[1] = a.y; acc[2] = a.z; acc[3] = a.w;
            acc[4] = b.x; acc[5] = b.y; acc[6] = b.z; acc[7] = b.w;
        }
        for (uint32_t r0 = 0; r0 < n_in; r0 += kSumBatch) {
            uint4 v[kSumBatch];
#pragma unroll
            for (uint32_t i = 0; i < kSumBatch; ++i)
                if (r0 + i < n_in) v[i] = ld_stream(static_cast<const uint4 *>(rp.p[r0 + i]) + c);
#pragma unroll
            for (uint32_t i = 0; i < kSumBatch; ++i) {
                if (r0 + i >= n_in) continue;
                const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
                const bool first = r0 + i == 0 && !accumulate;
#pragma unroll
                for (uint32_t e = 0; e < 8; ++e) {
                    const float x = __uint_as_float(e & 1u ? w[e >> 1] & 0xFFFF0000u : w[e >> 1] << 16);
                    acc[e] = first ? x : acc[e] + x;
                }
            }
        }
        st_stream(reinterpret_cast<float4 *>(out) + 2 * c, make_float4(acc[0], acc[1], acc[2], acc[3]));
        st_stream(reinterpret_cast<float4 *>(out) + 2 * c + 1,
                  make_float4(acc[4], acc[5], acc[6], acc[7]));
    }
    if (blockIdx.x == 0) {
        const uint32_t t = m8 * 8 + threadIdx.x;
        if (t < m) {
            float acc = accumulate ? out[t] : 0.0f;
            for (uint32_t r = 0; r < n_in; ++r) {
                const float x =
                    __uint_as_float(uint32_t(static_cast<const uint16_t *>(rp.p[r])[t]) << 16);
                acc = (r == 0 && !accumulate) ? x : acc + x;
            }
            out[t] = acc;
        }
    }
}

}  // namespace

int launch_encode(const tagc_plan_t *p, const tagc_rank_buffers *rk, const tagc_shared_buffers *sh,
                  hipStream_t s)
{
    ProfileScope ps("encode", s);
    const size_t lds = size_t(p->T_cap) * sizeof(float);
    static size_t attr_bytes = 0;
    if (lds > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(encode_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                int(lds)) != hipSuccess)
            return TAGC_EHIP;
        attr_bytes = lds;
    }
    encode_kernel<<<uint32_t(p->A_cap), kEncodeThreads, lds, s>>>(
        rk->idx, rk->val, rk->cnt, sh->header, rk->sketch, p->cfg.seed,
        sh->bounds + p->A_cap + 1, p->cnt_ranges, uint32_t(p->K),
        p->cfg.index_mode == TAGC_INDEX_OR1 ? nullptr : sh->bitmap,
        p->cfg.cell_type == TAGC_CELL_BF16);
    return hip_ok(hipGetLastError());
}

int launch_sketch_sum(const tagc_plan_t *p, const tagc_rank_buffers *ranks, uint32_t n_ranks,
                      const tagc_shared_buffers *sh, hipStream_t s)
{
    ProfileScope ps("sketch_sum", s);
    // one thread per float4 up to the plan's capacity; those beyond the m in the header leave
    const uint32_t grid = uint32_t(std::max<uint64_t>(1, (p->m_cap / 4 + 255) / 256));
    for (uint32_t r0 = 0; r0 < n_ranks; r0 += kMaxRanksPerPass) {
        RankPtrs rp{};
        const uint32_t n_in = std::min(kMaxRanksPerPass, n_ranks - r0);
        for (uint32_t r = 0; r < n_in; ++r) rp.p[r] = ranks[r0 + r].sketch;
        if (p->cfg.cell_type == TAGC_CELL_BF16)
            sketch_sum16_kernel<<<(grid + 1) / 2, 256, 0, s>>>(rp, n_in, sh->sketch, sh->header,
                                                                r0 != 0);
        else
            sketch_sum_kernel<<<grid, 256, 0, s>>>(rp, n_in, sh->sketch, sh->header, r0 != 0);
    }
    return hip_ok(hipGetLastError());
}

}  // namespace tagc
