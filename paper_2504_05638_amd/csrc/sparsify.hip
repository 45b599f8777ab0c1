// Stage 1 of the hot path: dynamic magnitude sparsifier + local Index.
//
// For every compressed segment of one rank's gradient bucket: find the threshold key T
// such that exactly k_l entries survive (section 3.2: the zeroing value is chosen
// dynamically so that at least theta of the values become zero), then emit the
// survivors as (c-index, float32 value) pairs in ascending c-index together with the
// 1-bit-per-parameter Index (Algorithm 1: sparsify, create_index).
//
// Keys: |g| as an unsigned integer (float32 bit pattern with the sign cleared; bf16 is
// widened first).  Ties at the threshold go to the lower position; exact zeros never
// survive.
//
// Two routes per segment, both exact:
//
//  candidate route (one read of the gradient)
//    prepare      only on the first call after the plan's table was uploaded: a strided
//                 sample gives every segment a conservative pre-threshold bin; afterwards
//                 each call leaves the pre-threshold for the next one in the table
//    scan_spill   streams the segment once: entries with key bin >= the pre-threshold
//                 ("candidates", ~1.3 x k of them) are histogrammed and spilled, in position
//                 order, into fixed slots per 4 KiB chunk -- no cross-wave dependency.  The
//                 workgroup that finishes a segment last selects its exact threshold from
//                 the candidate histogram; if the candidates do not contain k entries (the
//                 pre-threshold misled) the segment is re-routed
//    hist2c/select2  fp32 only: low 16 key bits inside the threshold bin
//    count        survivors of every super-chunk of candidates (32 chunks)
//    place        ordered pass over the candidates only: pairs + every Index word
//
//  dense route (segments that are short, unaligned, keep more than ~3 %, have no
//  pre-threshold yet, or were re-routed; three reads)
//    hist1        exact histogram of the top 15 key bits of every entry, in LDS; the
//                 workgroup that completes a segment's histogram selects its threshold
//    hist2/select2 fp32 only, as above
//    count        survivors of every tile of the gradient
//    place        ordered pass over the gradient: pairs + Index words
//
// count and place are one launch each for both routes.  Ordered output across workgroups
// needs no waiting: place starts when every count is there, and every item adds up the counts
// of the earlier items of its segment by itself.
//
// With a gradient accumulator (error feedback: Algorithm 1, lines 1-2) what is sparsified is
// grad + acc: scan_spill, and accumulate for the segments it does not read, write the sums
// back to acc, from which the dense route then reads; which of them were sent is recorded
// by the rank's own Index and applied when acc is read next (see SentMap).  With 4-bit
// counters on the wire (section 2.2) widen4 turns the Index into them at the end.
//
// Counters that must start at zero (arrivals, the candidate histograms) live in the plan's
// table, which only the library writes: whoever reads them last puts them back to zero, so
// no call spends a launch on clearing (see TableState).
#include <mutex>

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

__device__ inline uint32_t load_elem_bits(const char *base, uint64_t i, int dtype)
{
    if (dtype == kBF16) return uint32_t(reinterpret_cast<const uint16_t *>(base)[i]) << 16;
    return reinterpret_cast<const uint32_t *>(base)[i];
}

// float32 bit pattern of element e of a 16-byte vector
template <int DTYPE>
__device__ inline uint32_t vec_elem_bits(const uint32_t (&w)[4], uint32_t e)
{
    return DTYPE == kBF16 ? ((w[e >> 1] >> (16 * (e & 1))) << 16) : w[e];
}

// g + acc in the gradient's own type (Algorithm 1, line 1; section 3.2, local gradient
// accumulation): one float32 add per entry; a bf16 result is rounded to nearest-even (a NaN
// keeps a mantissa bit).  `g`, `a`: one 32-bit word of each buffer (two bf16 entries).
template <int DTYPE>
__device__ inline uint32_t sum_word(uint32_t g, uint32_t a)
{
    if (DTYPE == kF32) return __float_as_uint(__uint_as_float(g) + __uint_as_float(a));
    const float lo = __uint_as_float(g << 16) + __uint_as_float(a << 16);
    const float hi = __uint_as_float(g & 0xFFFF0000u) + __uint_as_float(a & 0xFFFF0000u);
    return round_to_bf16(lo) | (round_to_bf16(hi) << 16);
}
// the same for one entry given as float32 bit patterns; returns the entry's bit pattern in
// its own type (low 16 bits for bf16)
template <int DTYPE>
__device__ inline uint32_t sum_elem(uint32_t g_f32bits, uint32_t a_f32bits)
{
    const float x = __uint_as_float(g_f32bits) + __uint_as_float(a_f32bits);
    return DTYPE == kF32 ? __float_as_uint(x) : round_to_bf16(x);
}
__device__ inline void store_elem(char *base, uint64_t i, uint32_t bits, int dtype)
{
    if (dtype == kBF16) reinterpret_cast<uint16_t *>(base)[i] = uint16_t(bits);
    else reinterpret_cast<uint32_t *>(base)[i] = bits;
}

// Error feedback keeps the record of what a rank sent in the rank's Index, not in the
// accumulator: clearing ~1 % of the accumulator's entries one by one after the streaming
// pass touched almost half of its cache lines a second time (measured: 140 us per rank on
// 7B-shaped buckets).  Instead an entry of acc whose bit is set in the Index the rank's
// previous call left (`sent`: 1 bit per parameter, or the 4-bit counters) reads as 0, and
// the next call's streaming pass, which rewrites all of acc anyway, applies that.
struct SentMap {
    const uint32_t *map;  // the rank's Index buffer as the previous call left it
    uint32_t wire4;       // 4-bit counters instead of bits
};

// bit e <=> parameter ci + e was sent, for the VEC parameters of one 16-byte vector
// (ci a multiple of VEC, VEC = 4 or 8)
template <uint32_t VEC>
__device__ inline uint32_t sent_bits(const SentMap sm, uint32_t ci)
{
    if (sm.wire4) {
        const uint32_t w = sm.map[ci >> 3];
        return VEC == 8 ? nibbles_set(w) : nibbles_set((w >> (4 * (ci & 4u))) & 0xFFFFu);
    }
    const uint32_t b = reinterpret_cast<const uint8_t *>(sm.map)[ci >> 3];
    return VEC == 8 ? b : (b >> (ci & 4u)) & 0xFu;
}

__device__ inline bool sent_bit(const SentMap sm, uint32_t ci)
{
    if (sm.wire4) return ((sm.map[ci >> 3] >> (4 * (ci & 7u))) & 0xFu) != 0;
    return ((sm.map[ci >> 5] >> (ci & 31u)) & 1u) != 0;
}

// float32 bit pattern of entry i of a segment's accumulator, 0 if it was sent
__device__ inline uint32_t unsent_elem(const char *ab, uint64_t i, uint32_t c_off,
                                       const SentMap sm, int dtype)
{
    return sent_bit(sm, c_off + uint32_t(i)) ? 0u : load_elem_bits(ab, i, dtype);
}

// word j of an accumulator vector with the entries named by `bits` (see sent_bits) cleared
template <int DTYPE>
__device__ inline uint32_t unsent_word(uint32_t a, uint32_t bits, uint32_t j)
{
    if (DTYPE == kF32) return (bits >> j) & 1u ? 0u : a;
    const uint32_t two = (bits >> (2 * j)) & 3u;
    return a & ~((two & 1u ? 0xFFFFu : 0u) | (two & 2u ? 0xFFFF0000u : 0u));
}

// Error feedback for the segments scan_spill never streams (short, unaligned, keeping
// nothing or too much): acc <- grad + acc, entry by entry.  The dense route then reads its
// input from acc.  Workgroups stride over each such segment.
template <int DTYPE>
__global__ void __launch_bounds__(256)
accumulate_kernel(const char *__restrict__ grad, const uint32_t *__restrict__ table, char *acc,
                  const SentMap sent)
{
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    for (uint32_t l = 0; l < L; ++l) {
        const SegDev sd = segs[l];
        if (sd.n == 0 || (sd.flags & kSegFast)) continue;
        const char *gb = grad + sd.offset * EB;
        char *ab = acc + sd.offset * EB;
        const uint64_t stride = uint64_t(gridDim.x) * 256;
        if (sd.flags & kSegAligned) {
            const uint64_t nvec = sd.n / VEC;
            for (uint64_t v = uint64_t(blockIdx.x) * 256 + threadIdx.x; v < nvec; v += stride) {
                const uint4 g = ld_stream(reinterpret_cast<const uint4 *>(gb) + v);
                const uint4 a = ld_stream(reinterpret_cast<const uint4 *>(ab) + v);
                const uint32_t sb = sent_bits<VEC>(sent, sd.c_off + uint32_t(v) * VEC);
                reinterpret_cast<uint4 *>(ab)[v] =
                    make_uint4(sum_word<DTYPE>(g.x, unsent_word<DTYPE>(a.x, sb, 0)),
                               sum_word<DTYPE>(g.y, unsent_word<DTYPE>(a.y, sb, 1)),
                               sum_word<DTYPE>(g.z, unsent_word<DTYPE>(a.z, sb, 2)),
                               sum_word<DTYPE>(g.w, unsent_word<DTYPE>(a.w, sb, 3)));
            }
            if (blockIdx.x == 0) {
                const uint64_t i = nvec * VEC + threadIdx.x;
                if (i < sd.n)
                    store_elem(ab, i, sum_elem<DTYPE>(load_elem_bits(gb, i, DTYPE),
                                                      unsent_elem(ab, i, sd.c_off, sent, DTYPE)),
                               DTYPE);
            }
        } else {
            for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x; i < sd.n; i += stride)
                store_elem(ab, i, sum_elem<DTYPE>(load_elem_bits(gb, i, DTYPE),
                                                  unsent_elem(ab, i, sd.c_off, sent, DTYPE)),
                           DTYPE);
        }
    }
}

// ----------------------------------------------------------------- select

// Largest bin b with  sum_{x >= b} hist[x] >= need  (need >= 1).  1024 threads, thread t
// owns the BPT consecutive bins starting at t*BPT.  Returns false if the whole histogram
// holds fewer than `need`; *total_out is the histogram's sum either way.  A second count
// `need2` (0 = none) is located in the same pass: *bin2_out is the largest bin with at
// least need2 entries at or above it, or 0xFFFFFFFF if the histogram holds fewer.  So is,
// on request, the number of entries in the bins from `tail_from` upwards.  Bins below
// `floor_bin` count as empty.
template <int BPT>
__device__ inline bool select_bins(const uint32_t *hist, uint32_t need, uint32_t *bin_out,
                                   uint32_t *above_out, uint32_t *at_out, uint32_t *total_out,
                                   uint32_t *smem /* >= 24 words */, uint32_t need2 = 0,
                                   uint32_t *bin2_out = nullptr, uint32_t tail_from = 0,
                                   uint32_t *tail_out = nullptr, uint32_t floor_bin = 0)
{
    const uint32_t t = threadIdx.x;
    const uint4 *hv = reinterpret_cast<const uint4 *>(hist + uint64_t(t) * BPT);
    uint32_t bins[BPT];
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < BPT / 4; ++i) {
        const uint4 v = hv[i];
        bins[4 * i] = v.x; bins[4 * i + 1] = v.y; bins[4 * i + 2] = v.z; bins[4 * i + 3] = v.w;
    }
    // bins below `floor_bin` are read as empty (their counts are incomplete when part of the
    // scan ran with a higher pre-threshold)
#pragma unroll
    for (int b = 0; b < BPT; ++b) {
        if (t * BPT + b < floor_bin) bins[b] = 0;
        s += bins[b];
    }
    uint32_t total;
    uint32_t prefix = block_excl_scan<uint32_t, kHistThreads / 64>(s, &total, smem);
    uint32_t suffix = total - prefix;  // bins of this thread and all higher ones
    if (t == 0) {
        smem[19] = 0xFFFFFFFFu;
        smem[20] = 0;
    }
    __syncthreads();
    // entries in the bins from `tail_from` (a multiple of BPT) upwards, if asked for
    if (tail_out && t * BPT >= tail_from && s) atomicAdd(&smem[20], s);
    if (total >= need && suffix >= need && suffix - s < need) {
        uint32_t acc = suffix - s;
        bool done = false;
#pragma unroll
        for (int b = BPT - 1; b >= 0; --b) {
            const uint32_t c = bins[b];
            if (!done && acc + c >= need) {
                smem[16] = t * BPT + b;
                smem[17] = acc;
                smem[18] = c;
                done = true;
            }
            if (!done) acc += c;
        }
    }
    if (need2 && total >= need2 && suffix >= need2 && suffix - s < need2) {
        uint32_t acc = suffix - s;
        bool done = false;
#pragma unroll
        for (int b = BPT - 1; b >= 0; --b) {
            const uint32_t c = bins[b];
            if (!done && acc + c >= need2) {
                smem[19] = t * BPT + b;
                done = true;
            }
            if (!done) acc += c;
        }
    }
    __syncthreads();
    *bin_out = smem[16];
    *above_out = smem[17];
    *at_out = smem[18];
    *total_out = total;
    if (bin2_out) *bin2_out = smem[19];
    if (tail_out) *tail_out = smem[20];
    __syncthreads();
    return total >= need;
}

// The same for a workgroup of NT < 1024 threads (32768 bins: thread t owns the 32768 / NT
// consecutive bins from t * 32768 / NT), without the bins in registers: every thread adds up
// its bins as they stream by, and the one thread whose bins hold the answer reads them a
// second time from the top down.  For kernels that are launched on the off-chance and nearly
// always leave at once: what such a launch costs on a busy device is finding a compute unit
// with room for its workgroup, and four waves of few registers fit where sixteen do not.
template <uint32_t NT>
__device__ inline bool select_bins_streamed(const uint32_t *hist, uint32_t need, uint32_t *bin_out,
                                            uint32_t *above_out, uint32_t *at_out,
                                            uint32_t *total_out, uint32_t *smem /* >= 24 words */,
                                            uint32_t need2, uint32_t *bin2_out,
                                            uint32_t tail_from, uint32_t *tail_out)
{
    constexpr uint32_t BPT = kBins1 / NT;
    static_assert(BPT % 4 == 0 && BPT * NT == kBins1, "whole 16-byte groups of bins per thread");
    const uint32_t t = threadIdx.x;
    const uint4 *hv = reinterpret_cast<const uint4 *>(hist + uint64_t(t) * BPT);
    uint32_t s = 0;
    for (uint32_t i = 0; i < BPT / 4; ++i) {
        const uint4 v = hv[i];
        s += v.x + v.y + v.z + v.w;
    }
    uint32_t total;
    const uint32_t prefix = block_excl_scan<uint32_t, NT / 64>(s, &total, smem);
    const uint32_t suffix = total - prefix;  // bins of this thread and all higher ones
    if (t == 0) {
        smem[19] = 0xFFFFFFFFu;
        smem[20] = 0;
    }
    __syncthreads();
    if (tail_out && t * BPT >= tail_from && s) atomicAdd(&smem[20], s);
    // largest bin of this thread with at least `want` entries at or above it
    auto locate = [&](uint32_t want, uint32_t *bin, uint32_t *above, uint32_t *at) {
        uint32_t acc = suffix - s;
        for (int i = int(BPT / 4) - 1; i >= 0; --i) {
            const uint4 v = hv[i];
            const uint32_t c[4] = {v.x, v.y, v.z, v.w};
            for (int e = 3; e >= 0; --e) {
                if (acc + c[e] >= want) {
                    *bin = t * BPT + 4 * uint32_t(i) + uint32_t(e);
                    if (above) *above = acc;
                    if (at) *at = c[e];
                    return;
                }
                acc += c[e];
            }
        }
    };
    if (total >= need && suffix >= need && suffix - s < need)
        locate(need, &smem[16], &smem[17], &smem[18]);
    if (need2 && total >= need2 && suffix >= need2 && suffix - s < need2)
        locate(need2, &smem[19], nullptr, nullptr);
    __syncthreads();
    *bin_out = smem[16];
    *above_out = smem[17];
    *at_out = smem[18];
    *total_out = total;
    if (bin2_out) *bin2_out = smem[19];
    if (tail_out) *tail_out = smem[20];
    __syncthreads();
    return total >= need;
}

// ---------------------------------------------------------------- prepare

// First call after the table's upload (and plans without a scan to clear for them).  One
// workgroup per compressed segment: segments on the candidate route that have no
// pre-threshold yet get one from a strided sample of 16-byte vectors: the sample bin above
// which  k*S/n + 5*sqrt(k*S/n) + 16  sampled entries lie.  The margin makes it very unlikely
// that fewer than k entries of the whole segment pass the pre-threshold; if that still
// happens the selection notices and re-routes the segment.  A sample that holds too few
// non-zeros to say anything leaves the segment without one: it takes the dense route this
// time, whose histogram then provides it.  The remaining workgroups clear the histograms of
// the dense route when there is no scan to do it.
template <int DTYPE>
__global__ void __launch_bounds__(kHistThreads)
prepare_kernel(const char *__restrict__ grad, const char *acc, const SentMap sent,
               uint32_t *table, uint4 *zero_base, uint64_t zero_n16)
{
    extern __shared__ uint32_t h[];
    __shared__ uint32_t smem[32];
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    const uint32_t L = table[0];
    const uint32_t tid = threadIdx.x;
    if (blockIdx.x >= L) {
        const uint32_t fb = blockIdx.x - L, nfb = gridDim.x - L;
        const uint4 z = make_uint4(0, 0, 0, 0);
        for (uint64_t i = uint64_t(fb) * kHistThreads + tid; i < zero_n16;
             i += uint64_t(nfb) * kHistThreads)
            zero_base[i] = z;
        return;
    }
    const uint32_t l = blockIdx.x;
    const SegDev sd = reinterpret_cast<const SegDev *>(table + 8)[l];
    const TableState ts = table_state(table, L);
    if (sd.k == 0 || sd.n == 0 || !(sd.flags & kSegFast) || ts.hint[l]) return;
    for (uint32_t i = tid; i < kBins1; i += kHistThreads) h[i] = 0;
    __syncthreads();
    const uint32_t nvec = sd.n / VEC;
    const uint32_t S = min(nvec, kSampleVectors);
    const uint32_t stride = nvec / S;
    const uint4 *vp = reinterpret_cast<const uint4 *>(grad + sd.offset * EB);
    const uint4 *ap = acc ? reinterpret_cast<const uint4 *>(acc + sd.offset * EB) : nullptr;
    for (uint32_t i = tid; i < S; i += kHistThreads) {
        uint4 q = vp[uint64_t(i) * stride + (stride >> 1)];
        if (ap) {  // error feedback: what is sparsified is grad + acc
            const uint32_t v = i * stride + (stride >> 1);
            const uint4 a = ap[v];
            const uint32_t sb = sent_bits<VEC>(sent, sd.c_off + v * VEC);
            q = make_uint4(sum_word<DTYPE>(q.x, unsent_word<DTYPE>(a.x, sb, 0)),
                           sum_word<DTYPE>(q.y, unsent_word<DTYPE>(a.y, sb, 1)),
                           sum_word<DTYPE>(q.z, unsent_word<DTYPE>(a.z, sb, 2)),
                           sum_word<DTYPE>(q.w, unsent_word<DTYPE>(a.w, sb, 3)));
        }
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (uint32_t e = 0; e < VEC; ++e) {
            const uint32_t key = vec_elem_bits<DTYPE>(w, e) & 0x7FFFFFFFu;
            if (key) atomicAdd(&h[key >> 16], 1u);
        }
    }
    __syncthreads();
    const float ks = float(double(sd.k) * double(S * VEC) / double(sd.n));
    const uint32_t need = uint32_t(ks + 5.0f * sqrtf(ks) + 16.0f) + 1u;
    uint32_t bin, above, at, total;
    const bool found = select_bins<32>(h, need, &bin, &above, &at, &total, smem);
    // bin 0 (|g| < 2^-133) is never a candidate
    if (tid == 0 && found) ts.hint[l] = max(bin, 1u);
}

// ------------------------------------------------------------- scan_spill

// Streams every candidate-route segment once.  A wave owns one chunk (64 lanes x 4 rows
// of 16-byte vectors, contiguous) at a time; candidates (key bin >= binlo) are counted in
// the workgroup's LDS histogram and written in position order to the chunk's slot array.
// bf16 slot: (bf16 bits << 16) | position in chunk.  fp32 slot: value bits in cand[slot],
// position in cand[n_slots_total + slot].
//
// Work assignment: the chunks of all segments form one list (a segment's chunks start at
// its first super-chunk); each workgroup takes one contiguous span of it, its waves
// interleaved inside the span.  A workgroup therefore meets a segment boundary -- where
// the LDS histogram has to be flushed behind barriers -- only if its span straddles one,
// instead of the whole grid draining at every boundary.
//
// Memory operations of a wave complete, as far as the wave can tell, in the order they
// were issued, and a store is acknowledged later than a load returns: a wave that stores
// a chunk's slots and then loads the next chunk waits for the acknowledgement as well,
// about a microsecond per chunk.  So the steady state of this kernel issues loads only.
// The next chunk is requested while the current one is processed, and the slots of a
// dozen chunks pile up in the wave's LDS staging area and leave together (when the area
// is full, and at the end), at which point nothing is waiting behind the stores.
//
// Two 512-thread workgroups per CU.  With the next chunk always in flight that keeps about
// 32 MB of requests outstanding, enough to saturate HBM; more only lengthens the queue the
// last workgroups to start wait in, and they keep that lag to the end of the kernel.  The
// LDS pays for the chunk buffer (candidates are fetched from it by position instead of
// being selected out of sixteen registers) and the staging area.  The histogram covers the
// kWinBins bins from the segment's pre-threshold upwards (12 octaves of magnitude); what lies
// above them is only counted (it survives whenever the threshold is inside the window, and
// otherwise the segment is re-routed).  Slot order inside a chunk comes from a wave-local
// scan of the per-lane counts, so a wave never waits on another.
//
// A workgroup that is done with its part of a segment adds its histogram to the segment's
// in the plan's table and counts itself as arrived; the one that arrives last selects the
// segment's threshold on the spot (select_window) and puts the table words back to zero.
// The kernel's workgroups also clear, as they start, the dense route's histograms in the
// rank workspace, which nothing touches before the kernels after this one.
constexpr uint32_t kSpillThreads = 512;
#ifndef TAGC_SPILL_WGS
#define TAGC_SPILL_WGS 2
#endif
constexpr uint32_t kSpillWgsPerCU = TAGC_SPILL_WGS;  // workgroups launched per compute unit
constexpr uint32_t kSpillStage = 512;  // staged slots per wave
constexpr uint32_t kSpillList = 16;    // staged chunks per wave
constexpr uint32_t kWatchCalls = 8;    // calls that extrapolate a falling pre-threshold after a miss
constexpr uint32_t kSpillRaise = 6;    // bins (1/128 octave each) a wave's pre-threshold goes up per try

// Threshold of one candidate-route segment from its candidate histogram `win` (table), by
// the kSpillThreads threads of the scan's last workgroup on the segment.  Leaves SelDev,
// the segment's count, the pre-threshold for the next call, and the table words at zero.
// pre-threshold for the next call from `bin2`, the bin above which 1.3 k entries lie now:
// that bin itself, or, in the calls after a miss (the scale fell by more than the margin
// since the hint was tuned), lower by the factor it fell by since the call before (at most
// half an octave) and 1.5 % more.  Bins are float32 bit patterns >> 16: the magnitudes are
// extrapolated, not the bin numbers, whose width in relative terms varies twofold across an
// octave.
__device__ inline uint32_t next_hint(uint32_t bin2, uint32_t prev, uint32_t watch)
{
    if (!watch || prev <= bin2) return max(bin2, 1u);
    const float now = __uint_as_float(bin2 << 16), before = __uint_as_float(prev << 16);
    const float fall = fmaxf(now / before, 0.7071f);
    return max(__float_as_uint(now * fall * 0.985f) >> 16, 1u);
}

template <int DTYPE>
__device__ inline void select_window(uint32_t l, const SegDev &sd, uint32_t blo,
                                     const TableState ts, SelDev *sel, uint32_t *smem /* >= 32 */)
{
    constexpr uint32_t BPT = kWinBins / kSpillThreads;  // consecutive bins per thread
    static_assert(BPT * kSpillThreads == kWinBins, "every thread owns BPT bins of the window");
    const uint32_t tid = threadIdx.x;
    uint32_t *win = ts.win + size_t(l) * kWinWords;
    uint32_t c[BPT];
#pragma unroll
    for (uint32_t b = 0; b < BPT; ++b) {
        c[b] = win[tid * BPT + b];
        win[tid * BPT + b] = 0;
    }
    const uint32_t above_w = win[kWinBins], nf = win[kWinBins + 1];
    const uint32_t raised = ts.raised[l], overflow = ts.reroute[l];
    const uint32_t prev = ts.prev[l], wt = ts.watch[l];  // (requested with the rest)
    __syncthreads();  // everybody has read what thread 0 clears next
    if (tid == 0) {
        win[kWinBins] = win[kWinBins + 1] = 0;
        ts.raised[l] = ts.reroute[l] = ts.arrive[l] = 0;
    }
    // the histogram is complete from the highest pre-threshold any wave used upwards
    const uint32_t floor_bin = max(blo, raised), floor_w = floor_bin - blo;
    uint32_t s = 0;
#pragma unroll
    for (uint32_t b = 0; b < BPT; ++b) {
        if (tid * BPT + b < floor_w) c[b] = 0;
        s += c[b];
    }
    uint32_t total;
    const uint32_t prefix = block_excl_scan<uint32_t, kSpillThreads / 64>(s, &total, smem);
    const uint32_t suffix = total - prefix + above_w;  // this thread's bins and everything higher
    // largest bin with at least `need` entries at or above it; twice: the threshold (k), and
    // the pre-threshold for the next call (1.3 k, what the slots per chunk are sized for)
    const uint32_t want = uint32_t(1.3f * float(sd.k)) + 1u;
    if (tid == 0) smem[16] = smem[19] = 0xFFFFFFFFu;
    __syncthreads();
    auto locate = [&](uint32_t need, uint32_t *bin_out, uint32_t *above_out) {
        if (!(s && suffix >= need && suffix - s < need)) return;
        uint32_t acc = suffix - s;  // entries in the bins above the one looked at
#pragma unroll
        for (int b = int(BPT) - 1; b >= 0; --b) {
            if (acc + c[b] >= need) {
                *bin_out = tid * BPT + uint32_t(b);
                if (above_out) *above_out = acc;
                return;
            }
            acc += c[b];
        }
    };
    locate(sd.k, &smem[16], &smem[17]);
    locate(want, &smem[19], nullptr);
    __syncthreads();
    if (tid != 0) return;
    const uint32_t bin_w = smem[16], above = smem[17], bin2_w = smem[19];
    const bool found = bin_w != 0xFFFFFFFFu && !overflow && blo != 0;
    SelDev r{};
    if (!found) {
        // The candidates hold fewer than k entries (the scale fell since the pre-threshold
        // was tuned), the threshold lies above the window, slots overflowed, or there was no
        // pre-threshold: dense route, whose histogram also provides the next pre-threshold.
        r.route = 1;
        if (blo != 0 && !overflow && above_w < sd.k) ts.watch[l] = kWatchCalls;
        ts.hint[l] = 0;
        sel[l] = r;
        return;
    }
    // The window may not reach down to 1.3 k entries; then one bin below what this call
    // could see.
    const uint32_t bin2 = bin2_w != 0xFFFFFFFFu ? max(blo + bin2_w, 1u) : max(floor_bin, 2u) - 1u;
    ts.hint[l] = next_hint(bin2, prev, wt);
    ts.prev[l] = bin2;
    if (wt) ts.watch[l] = wt - 1;
    if (nf) atomicAdd(&ts.glob[1], nf);
    const uint32_t T_bin = blo + bin_w;
    if (DTYPE == kBF16) {
        r.T = T_bin << 16;
        r.G = above;
        r.quota = sd.k - above;
        r.cnt = sd.k;
    } else {
        r.bin1 = T_bin;
        r.G1 = above;
        r.need2 = 1;
    }
    sel[l] = r;
}

template <int DTYPE>
__global__ void __launch_bounds__(kSpillThreads)
scan_spill_kernel(const char *__restrict__ grad, char *acc, const SentMap sent,
                  uint32_t *table, SelDev *sel, uint32_t *__restrict__ cand,
                  uint2 *__restrict__ chunk_info, uint64_t n_slots_total, uint32_t CAP,
                  uint4 *zero_base, uint64_t zero_n16)
{
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    constexpr uint32_t ROWS = kCandRows;
    constexpr uint32_t ROW_ELEMS = 64 * VEC;
    constexpr uint32_t CHUNK = ROW_ELEMS * ROWS;
    constexpr uint32_t NW = kSpillThreads / 64;
    constexpr uint32_t STAGE_WORDS = kSpillStage * (DTYPE == kBF16 ? 1 : 2);
    static_assert(ROWS == 4 && ROWS * VEC <= 32, "packed masks and row counts below");
    __shared__ uint32_t h[kWinWords];
    __shared__ uint32_t s_sel[32];
    __shared__ uint32_t s_last;
    __shared__ uint32_t s_region;  // slots of the workgroup's part of `cand` handed out so far
    __shared__ uint32_t stage[NW][STAGE_WORDS];
    __shared__ uint32_t list[NW][3][kSpillList];  // chunk number, staging offset, count
    __shared__ uint4 data[NW][ROWS * 64];         // each wave's current chunk
    const uint32_t L = table[0];
    const uint32_t total_chunks = table[4] * kCandChunksPerSuper;
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const TableState ts = table_state(table, L);
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    // wave-uniform by construction; saying so keeps chunk addresses in scalar registers
    const uint32_t wib = __builtin_amdgcn_readfirstlane(tid >> 6);
    {   // the dense route's histograms start at zero (nobody reads them before this kernel ends)
        const uint4 z = make_uint4(0, 0, 0, 0);
        for (uint64_t i = uint64_t(blockIdx.x) * kSpillThreads + tid; i < zero_n16;
             i += uint64_t(gridDim.x) * kSpillThreads)
            zero_base[i] = z;
    }
    uint32_t span = (total_chunks + gridDim.x - 1) / gridDim.x;
    span = (span + NW - 1) / NW * NW;
    const uint64_t g0 = uint64_t(blockIdx.x) * span;
    if (g0 >= total_chunks) return;
    const uint64_t g1 = min(g0 + span, uint64_t(total_chunks));
    for (uint32_t i = tid; i < kWinWords; i += kSpillThreads) h[i] = 0;
    if (tid == 0) s_region = 0;
    // last segment whose first chunk is not beyond the span's start.  Up to 64 segments: lane
    // i looks at segment i, all at once (a search would be several dependent loads, which is
    // time the workgroup's first chunk waits for)
    uint32_t l0 = 0;
    if (L <= 64) {
        const uint64_t first = lane < L ? uint64_t(segs[lane].sc_start) * kCandChunksPerSuper
                                        : ~0ull;
        l0 = uint32_t(__popcll(__ballot(first <= g0))) - 1u;  // segment 0 starts at chunk 0
    } else {
        for (uint32_t hi = L; hi - l0 > 1;) {
            const uint32_t mid = (l0 + hi) >> 1;
            if (uint64_t(segs[mid].sc_start) * kCandChunksPerSuper <= g0) l0 = mid;
            else hi = mid;
        }
    }
    __syncthreads();  // h[] is clear
    uint32_t *st = stage[wib];
    uint32_t *lst_chunk = list[wib][0], *lst_off = list[wib][1], *lst_cnt = list[wib][2];
    uint4 *dw = data[wib];
    const bool staged = CAP <= kSpillStage;
    uint32_t n_list = 0, fill = 0;  // wave-uniform

    // The staged chunks' slots and counts go out; only this wave touched what it reads.
    // The slots are packed: the chunks of the workgroup's span own the part
    // [g0 * CAP, g1 * CAP) of `cand`, and every flush takes the next free stretch of it, a
    // whole number of 128-byte lines (a line written only in part costs the memory system a
    // read-modify-write; a stretch never needs more than its chunks' CAP slots each, so the
    // part cannot run out).  Where a chunk's slots went is recorded beside its count.  With
    // one fixed array of CAP slots per chunk, of which a quarter is used on average, every
    // pass over the slots moved twice the bytes.
    auto flush = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint32_t n_out = (fill + 31u) & ~31u;
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(&s_region, n_out);
        at = __builtin_amdgcn_readfirstlane(at);
        const uint32_t first = uint32_t(g0) * CAP + at;  // (the plan keeps slot numbers in 32 bits)
        uint32_t *slots = cand + first;
        // the padding words are stale staging content, which no reader looks at
        for (uint32_t i = lane; i < n_out; i += 64) {
            slots[i] = st[i];
            if (DTYPE != kBF16) slots[n_slots_total + i] = st[kSpillStage + i];
        }
        if (lane < n_list)
            chunk_info[lst_chunk[lane]] = make_uint2(lst_cnt[lane], first + lst_off[lane]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        n_list = 0;
        fill = 0;
    };

    for (uint32_t l = l0; l < L; ++l) {
        const SegDev sd = segs[l];
        const uint64_t s0 = uint64_t(sd.sc_start) * kCandChunksPerSuper;
        if (s0 >= g1) break;
        if (sd.k == 0 || sd.n == 0 || !(sd.flags & kSegFast)) continue;
        const uint32_t n_chunks = (sd.n + CHUNK - 1) / CHUNK;
        const uint32_t lo = g0 > s0 ? uint32_t(g0 - s0) : 0u;
        const uint32_t hi = uint32_t(min(uint64_t(n_chunks), g1 - s0));
        if (lo >= hi) continue;
        // No pre-threshold (the sample could not tell, or the last call withdrew it): the
        // segment takes the dense route this time.
        // With an accumulator (error feedback) the segment is streamed all the same: this
        // pass is also the one that turns acc into grad + acc, which the dense route then
        // reads instead of the gradient.  Its candidates are then never used.
        const uint32_t hint = ts.hint[l];
        const uint32_t blo = hint ? hint : 0x7F7Fu;  // 1 <= blo <= 0x7FFF
        if (hint || acc) {
            const char *base = grad + sd.offset * EB;
            char *abase = acc ? acc + sd.offset * EB : nullptr;
            // The wave's own pre-threshold: starts at the segment's and goes up when a chunk
            // holds more candidates than it has slots (see below).
            uint32_t blo_w = blo, swar_add = (0x8000u - blo) * 0x10001u;
            bool overflow = false;
            // the lane's four vectors of chunk `ch`; entries past the segment's end read as 0
            auto load_chunk = [&](const char *base, uint32_t ch, uint32_t (&w)[ROWS][4]) {
                const uint32_t rel0 = ch * CHUNK;
                if (rel0 + CHUNK <= sd.n) {
                    const uint4 *q = reinterpret_cast<const uint4 *>(base + uint64_t(rel0) * EB) + lane;
#pragma unroll
                    for (uint32_t r = 0; r < ROWS; ++r) {
                        const uint4 v = ld_stream(q + 64 * r);  // read once, never again
                        w[r][0] = v.x; w[r][1] = v.y; w[r][2] = v.z; w[r][3] = v.w;
                    }
                } else {
#pragma unroll
                    for (uint32_t r = 0; r < ROWS; ++r) {
                        const uint32_t rel = rel0 + r * ROW_ELEMS + lane * VEC;
                        w[r][0] = w[r][1] = w[r][2] = w[r][3] = 0;
                        if (rel + VEC <= sd.n) {
                            const uint4 v = *reinterpret_cast<const uint4 *>(base + uint64_t(rel) * EB);
                            w[r][0] = v.x; w[r][1] = v.y; w[r][2] = v.z; w[r][3] = v.w;
                        } else if (rel < sd.n) {
#pragma unroll
                            for (uint32_t e = 0; e < VEC; ++e) {
                                if (rel + e >= sd.n) continue;
                                const uint32_t b = load_elem_bits(base, uint64_t(rel) + e, DTYPE);
                                if (DTYPE == kBF16) w[r][e >> 1] |= (b >> 16) << (16 * (e & 1));
                                else w[r][e] = b;
                            }
                        }
                    }
                }
            };
            // The sums of chunk `ch` back to the accumulator (entries inside the segment only),
            // from the chunk's LDS copy: the stores are issued after the next chunk's loads,
            // whose registers the sums no longer occupy, so that waiting for those loads does
            // not mean waiting for the stores' acknowledgements as well.
            auto store_chunk = [&](uint32_t ch) {
                const uint32_t rel0 = ch * CHUNK;
                if (rel0 + CHUNK <= sd.n) {
                    uint4 *q = reinterpret_cast<uint4 *>(abase + uint64_t(rel0) * EB) + lane;
#pragma unroll
                    for (uint32_t r = 0; r < ROWS; ++r) st_stream(q + 64 * r, dw[r * 64 + lane]);
                } else {
#pragma unroll
                    for (uint32_t r = 0; r < ROWS; ++r) {
                        const uint32_t rel = rel0 + r * ROW_ELEMS + lane * VEC;
                        const uint4 v = dw[r * 64 + lane];
                        const uint32_t x[4] = {v.x, v.y, v.z, v.w};
                        if (rel + VEC <= sd.n) {
                            *reinterpret_cast<uint4 *>(abase + uint64_t(rel) * EB) = v;
                        } else if (rel < sd.n) {
#pragma unroll
                            for (uint32_t e = 0; e < VEC; ++e) {
                                if (rel + e >= sd.n) continue;
                                const uint32_t b = DTYPE == kBF16
                                                       ? (x[e >> 1] >> (16 * (e & 1))) & 0xFFFFu
                                                       : x[e];
                                store_elem(abase, uint64_t(rel) + e, b, DTYPE);
                            }
                        }
                    }
                }
            };
            // which of the lane's accumulator entries of chunk `ch` the previous call sent
            // (one byte or half a byte of the 1-bit Index per vector, one word or half a
            // word of the 4-bit one); vectors past the segment's end have none
            auto load_sent = [&](uint32_t ch, uint32_t (&sb)[ROWS]) {
#pragma unroll
                for (uint32_t r = 0; r < ROWS; ++r) {
                    const uint32_t rel = ch * CHUNK + r * ROW_ELEMS + lane * VEC;
                    sb[r] = rel < sd.n ? sent_bits<VEC>(sent, sd.c_off + rel) : 0u;
                }
            };
            uint32_t w[ROWS][4], aw[ROWS][4], sb[ROWS];
            if (lo + wib < hi) {
                load_chunk(base, lo + wib, w);
                if (acc) {
                    load_chunk(abase, lo + wib, aw);
                    load_sent(lo + wib, sb);
                }
            }
            for (uint32_t ch = lo + wib; ch < hi; ch += NW) {
                if (acc) {  // error feedback: sparsify grad + acc, and keep the sums
#pragma unroll
                    for (uint32_t r = 0; r < ROWS; ++r)
#pragma unroll
                        for (uint32_t j = 0; j < 4; ++j)
                            w[r][j] = sum_word<DTYPE>(w[r][j], unsent_word<DTYPE>(aw[r][j], sb[r], j));
                }
                // Keep the chunk in LDS (a lane only ever reads back what it wrote itself).
                // Branch-free classification: bit r*VEC + e of `mask` <=> entry e of the
                // lane's vector in row r is a candidate.
                uint32_t mask = 0, c[ROWS];
#pragma unroll
                for (uint32_t r = 0; r < ROWS; ++r) {
                    dw[r * 64 + lane] = make_uint4(w[r][0], w[r][1], w[r][2], w[r][3]);
                    uint32_t f = 0;
                    if (DTYPE == kBF16) {
                        // both halves of a word at once: adding 0x8000 - binlo to a 15-bit
                        // key sets bit 15 exactly when key >= binlo, without carrying over
#pragma unroll
                        for (uint32_t j = 0; j < 4; ++j) {
                            const uint32_t t = ((w[r][j] & 0x7FFF7FFFu) + swar_add) & 0x80008000u;
                            f |= (t >> 15) << (2 * j);  // low half -> bit 2j, high -> bit 2j+16
                        }
                        c[r] = __popc(f);
                        f = (f & 0xFFFFu) | ((f >> 16) << 1);
                    } else {
#pragma unroll
                        for (uint32_t e = 0; e < VEC; ++e)
                            f |= uint32_t(((w[r][e] & 0x7FFFFFFFu) >> 16) >= blo_w) << e;
                        c[r] = __popc(f);
                    }
                    mask |= f << (r * VEC);
                }
                if (ch + NW < hi) {  // in flight during the rest
                    load_chunk(base, ch + NW, w);
                    if (acc) {
                        load_chunk(abase, ch + NW, aw);
                        load_sent(ch + NW, sb);
                    }
                }
                if (acc) store_chunk(ch);
                // slot of each lane's first candidate per row: one scan over the four
                // row counts packed in 16-bit fields (a row holds at most 512 candidates)
                uint32_t p01, p23, total;
                auto place = [&]() {
                    const uint32_t ia = wave_incl_scan<uint32_t>(c[0] | (c[1] << 16));
                    const uint32_t ib = wave_incl_scan<uint32_t>(c[2] | (c[3] << 16));
                    const uint32_t ta = __builtin_amdgcn_readlane(ia, 63);
                    const uint32_t tb = __builtin_amdgcn_readlane(ib, 63);
                    const uint32_t t0 = ta & 0xFFFFu, t1 = ta >> 16, t2 = tb & 0xFFFFu,
                                   t3 = tb >> 16;
                    // exclusive positions, again two per register: rows 0,1 and rows 2,3
                    p01 = ia - (c[0] | (c[1] << 16)) + (t0 << 16);
                    p23 = ib - (c[2] | (c[3] << 16)) + (t0 + t1) * 0x10001u + (t2 << 16);
                    total = t0 + t1 + t2 + t3;
                };
                place();
                // More candidates than the chunk has slots: the pre-threshold this call was
                // given is too low (the gradient's scale went up since it was tuned; with
                // error feedback it does every step).  Rather than giving the segment up to
                // the two-read route, the wave raises its own pre-threshold -- for this chunk,
                // classified again from its LDS copy, and for the chunks it takes after it --
                // until the chunk fits.  Nothing has been counted or stored for the chunk yet.
                // The highest pre-threshold any wave used is recorded: the histogram is only
                // complete from there upwards, which is where the selection then looks.
                while (total > CAP && blo_w < 0x7F7Fu) {
                    blo_w = min(blo_w + kSpillRaise, 0x7F7Fu);
                    swar_add = (0x8000u - blo_w) * 0x10001u;
                    mask = 0;
#pragma unroll
                    for (uint32_t r = 0; r < ROWS; ++r) {
                        const uint4 v = dw[r * 64 + lane];
                        const uint32_t x[4] = {v.x, v.y, v.z, v.w};
                        uint32_t f = 0;
                        if (DTYPE == kBF16) {
#pragma unroll
                            for (uint32_t j = 0; j < 4; ++j) {
                                const uint32_t t = ((x[j] & 0x7FFF7FFFu) + swar_add) & 0x80008000u;
                                f |= (t >> 15) << (2 * j);
                            }
                            c[r] = __popc(f);
                            f = (f & 0xFFFFu) | ((f >> 16) << 1);
                        } else {
#pragma unroll
                            for (uint32_t e = 0; e < VEC; ++e)
                                f |= uint32_t(((x[e] & 0x7FFFFFFFu) >> 16) >= blo_w) << e;
                            c[r] = __popc(f);
                        }
                        mask |= f << (r * VEC);
                    }
                    place();
                }
                const uint32_t chunk_id = uint32_t(s0) + ch;
                // (a chunk's slots start on a 16-byte boundary: they are read in such groups)
                const uint32_t need = min((total + 3u) & ~3u, CAP);
                if (staged && (n_list == kSpillList || fill + need > kSpillStage)) flush();
                uint32_t *slots = cand + uint64_t(chunk_id) * CAP;
                uint32_t *slots_pos = slots + n_slots_total;  // fp32 only
                uint32_t *stc = st + fill;
                // Candidates are rare: every lane walks its own few set bits, so the wave
                // issues as many histogram / store instructions as its busiest lane needs.
                for (uint32_t mm = mask; mm;) {
                    const uint32_t e = __builtin_ctz(mm);
                    mm &= mm - 1;
                    const uint32_t r = e / VEC;
                    const uint32_t row_bits = ((1u << VEC) - 1u) << (r * VEC);
                    const uint32_t before = __popc(mask & row_bits & ((1u << e) - 1u));
                    const uint32_t ps = (((r & 2u) ? p23 : p01) >> (16 * (r & 1u)) & 0xFFFFu) + before;
                    const uint32_t rel = r * ROW_ELEMS + lane * VEC + (e % VEC);
                    uint32_t bits;
                    if (DTYPE == kBF16)
                        bits = uint32_t(reinterpret_cast<const uint16_t *>(dw)[rel]) << 16;
                    else
                        bits = reinterpret_cast<const uint32_t *>(dw)[rel];
                    const uint32_t bin = (bits & 0x7FFFFFFFu) >> 16;
                    atomicAdd(&h[min(bin - blo, kWinBins)], 1u);      // in the window, or above it
                    if (bin >= 0x7F80u) atomicAdd(&h[kWinBins + 1], 1u);  // all-ones exponent
                    if (ps < CAP) {
                        if (DTYPE == kBF16) {
                            if (staged) stc[ps] = bits | rel;
                            else slots[ps] = bits | rel;
                        } else {
                            if (staged) {
                                stc[ps] = bits;
                                stc[kSpillStage + ps] = rel;
                            } else {
                                slots[ps] = bits;
                                slots_pos[ps] = rel;
                            }
                        }
                    }
                }
                if (staged) {
                    if (lane == 0) {
                        lst_chunk[n_list] = chunk_id;
                        lst_off[n_list] = fill;
                        lst_cnt[n_list] = total;
                    }
                    ++n_list;
                    fill += need;
                } else if (lane == 0) {
                    chunk_info[chunk_id] = make_uint2(total, chunk_id * CAP);
                }
                overflow |= total > CAP;
            }
            if (staged && n_list) flush();
            if (blo_w > blo && lane == 0) atomicMax(&ts.raised[l], blo_w);
            if (overflow && lane == 0)  // a chunk denser than its slots: take the dense route
                atomicOr(&ts.reroute[l], 1u);
        }
        __syncthreads();
        uint32_t *win = ts.win + size_t(l) * kWinWords;
        for (uint32_t i = tid; i < kWinWords; i += kSpillThreads) {
            const uint32_t c = h[i];
            if (c) {
                atomicAdd(&win[i], c);
                h[i] = 0;
            }
        }
        // The table updates are device-scope atomics, performed where every CU sees them; a
        // thread only has to wait until its own have been acknowledged before the workgroup
        // counts as arrived.  The workgroup that arrives last drops what it may hold of the
        // table in its caches and selects.
        wait_own_memory_ops();
        __syncthreads();
        if (tid == 0) {
            const uint64_t c_last = s0 + n_chunks - 1;  // segment's chunks: one workgroup per span
            const uint32_t expected = uint32_t(c_last / span) - uint32_t(s0 / span) + 1u;
            s_last = atomicAdd(&ts.arrive[l], 1u) == expected - 1u;
        }
        __syncthreads();
        if (s_last) {  // uniform
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            select_window<DTYPE>(l, sd, hint, ts, sel, s_sel);
        }
        __syncthreads();
    }
}

// Whether segment l is on the dense route: by plan (not eligible for the candidate route), or
// because the scan's selection sent it there (no pre-threshold, too few candidates, a chunk
// denser than its slots).  sel[l] of a candidate-route segment has been written by the scan.
__device__ inline bool on_dense_route(const SegDev &sd, const SelDev *sel, uint32_t l)
{
    if (sd.k == 0 || sd.n == 0) return false;
    return !(sd.flags & kSegFast) || sel[l].route != 0;
}

// true iff some segment is on the dense route.  Every thread reads the same words, so the
// loads are scalar and the answer is uniform without a barrier.
__device__ inline bool any_dense_route(const SegDev *segs, const SelDev *sel, uint32_t L)
{
    bool any = false;
    for (uint32_t l = 0; l < L; ++l) any |= on_dense_route(segs[l], sel, l);
    return any;
}

// ------------------------------------------------------------------ hist1

// LDS histogram of the dense route: `WBINS` counters for the bins from `base` upwards; an
// entry outside that window goes straight to the global histogram `gh`.
template <uint32_t WBINS>
struct HistWin {
    uint32_t *h, *gh;
    uint32_t base;
    __device__ inline void add(uint32_t bin) const
    {
        if (WBINS == kBins1) {
            atomicAdd(&h[bin], 1u);
        } else {
            const uint32_t wi = bin - base;
            if (wi < WBINS) atomicAdd(&h[wi], 1u);
            else atomicAdd(&gh[bin], 1u);
        }
    }
};

template <int DTYPE, uint32_t WBINS>
__device__ inline void hist_word(uint32_t w, const HistWin<WBINS> &hw)
{
    if (DTYPE == kBF16) {
        uint32_t a = w & 0x7FFFu, b = (w >> 16) & 0x7FFFu;
        if (a) hw.add(a);
        if (b) hw.add(b);
    } else {
        uint32_t key = w & 0x7FFFFFFFu;
        if (key) hw.add(key >> 16);
    }
}

template <int DTYPE, uint32_t WBINS>
__device__ inline void hist_vec(uint4 v, const HistWin<WBINS> &hw)
{
    hist_word<DTYPE>(v.x, hw);
    hist_word<DTYPE>(v.y, hw);
    hist_word<DTYPE>(v.z, hw);
    hist_word<DTYPE>(v.w, hw);
}

template <uint32_t WBINS>
__device__ inline void hist_elem(uint32_t f32bits, const HistWin<WBINS> &hw)
{
    uint32_t key = f32bits & 0x7FFFFFFFu;
    if (key) hw.add(key >> 16);
}

// Threshold bin of one dense-route segment from the 32768-bin histogram of all its entries,
// by a whole workgroup of NT threads.  Also leaves the pre-threshold for the next
// call on this plan: the bin above which about 1.3 k entries lie (what the slots per chunk
// are sized for).
template <int DTYPE, uint32_t NT>
__device__ inline void select_dense(uint32_t l, const SegDev &sd, const uint32_t *hist,
                                    SelDev *sel, const TableState ts,
                                    uint32_t *smem /* >= 32 words */)
{
    const uint32_t *h = hist + uint64_t(l) * kBins1;
    uint32_t bin, above, at, total, bin2, nf;
    const bool fast = (sd.flags & kSegFast) != 0;
    const uint32_t want = fast ? uint32_t(1.3f * float(sd.k)) + 1u : 0u;
    // nf: inputs with an all-ones exponent fall into bins >= 0x7F80
    const bool found =
        NT == kHistThreads
            ? select_bins<32>(h, sd.k, &bin, &above, &at, &total, smem, want, &bin2, 0x7F80u, &nf)
            : select_bins_streamed<NT>(h, sd.k, &bin, &above, &at, &total, smem, want, &bin2,
                                       0x7F80u, &nf);
    if (threadIdx.x != 0) return;
    if (fast) {
        // fewer non-zeros than 1.3 k in the whole segment: everything is a candidate
        const uint32_t b2 = bin2 != 0xFFFFFFFFu ? max(bin2, 1u) : 1u;
        // after a miss (the scale fell below what the carried pre-threshold admits) the next
        // calls extrapolate the fall instead of trusting the last value
        ts.hint[l] = next_hint(b2, ts.prev[l], ts.watch[l]);
        ts.prev[l] = b2;
    }
    if (nf) atomicAdd(&ts.glob[1], nf);
    atomicAdd(&ts.glob[2], 1u);
    SelDev r{};
    r.route = 1;
    if (!found) {  // fewer non-zeros than k: keep every non-zero
        r.T = 0;
        r.quota = 0;
        r.G = total;
        r.cnt = total;
    } else if (DTYPE == kBF16) {
        r.T = bin << 16;
        r.G = above;
        r.quota = sd.k - above;
        r.cnt = sd.k;
    } else {
        r.bin1 = bin;
        r.G1 = above;
        r.need2 = 1;
    }
    sel[l] = r;
}

// Dense route: one workgroup per CU, all entries of every dense-route segment.  Leaves at
// once when no segment is on the dense route.  The workgroup that completes a segment's
// histogram selects its threshold right away, while the others go on with the next segment:
// no separate selection launch.
//
// WBINS = 32768: all counters in LDS (128 KiB), for plans with dense-route segments.  A plan
// without any launches the kernel only as the safety net of re-routed segments, and a
// workgroup that needs most of a compute unit's LDS has to wait, on a busy device, until
// one is that free -- just to find that there is nothing to do.  Such plans use WBINS = 4096
// (16 KiB): the 32 octaves around the segment's last pre-threshold, where all but a
// vanishing part of a gradient lies; the rest is added to the global histogram directly.
// And workgroups of 256 threads, four per CU: with buckets in flight on other streams a
// 1024-thread workgroup found room 7 us later on average, per rank and bucket, 3.3 ms per
// step of the 7B workload -- for a launch that reads two table rows and leaves.
constexpr uint32_t kHistWindow = 4096;
constexpr uint32_t kHistNetThreads = 256;

template <int DTYPE, uint32_t WBINS, uint32_t NT>
__global__ void __launch_bounds__(NT)
hist1_kernel(const char *__restrict__ grad, uint32_t *table, SelDev *sel, uint32_t *hist)
{
    extern __shared__ uint32_t h[];
    __shared__ uint32_t s_sel[32];
    __shared__ uint32_t s_last;
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    if (!any_dense_route(segs, sel, L)) return;
    const TableState ts = table_state(table, L);
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < WBINS; i += NT) h[i] = 0;
    __syncthreads();
    for (uint32_t l = 0; l < L; ++l) {
        const SegDev sd = segs[l];
        if (!on_dense_route(sd, sel, l)) continue;
        const char *base = grad + sd.offset * EB;
        uint32_t *gh = hist + uint64_t(l) * kBins1;
        // window: 24 octaves below to 8 above the bin the last call's 1.3 k largest entries
        // began at; without one, magnitudes from 2^-30 to 4
        const uint32_t prev = ts.prev[l];
        const HistWin<WBINS> hw{h, gh, WBINS == kBins1 ? 0u
                                          : (prev ? (prev > 3072u ? min(prev - 3072u, kBins1 - WBINS) : 0u)
                                                  : 97u * 128u)};
        if (sd.flags & kSegAligned) {
            const uint4 *vp = reinterpret_cast<const uint4 *>(base);
            const uint64_t nvec = sd.n / VEC;
            const uint64_t stride = uint64_t(gridDim.x) * NT;
            uint64_t v = uint64_t(blockIdx.x) * NT + tid;
            for (; v + 3 * stride < nvec; v += 4 * stride) {
                const uint4 a = ld_stream(vp + v), b = ld_stream(vp + v + stride),
                            c = ld_stream(vp + v + 2 * stride), d = ld_stream(vp + v + 3 * stride);
                hist_vec<DTYPE>(a, hw);
                hist_vec<DTYPE>(b, hw);
                hist_vec<DTYPE>(c, hw);
                hist_vec<DTYPE>(d, hw);
            }
            for (; v < nvec; v += stride) hist_vec<DTYPE>(ld_stream(vp + v), hw);
            if (blockIdx.x == 0) {
                uint64_t i = nvec * VEC + tid;
                if (i < sd.n) hist_elem(load_elem_bits(base, i, DTYPE), hw);
            }
        } else {
            for (uint64_t i = uint64_t(blockIdx.x) * NT + tid; i < sd.n;
                 i += uint64_t(gridDim.x) * NT)
                hist_elem(load_elem_bits(base, i, DTYPE), hw);
        }
        __syncthreads();
        for (uint32_t i = tid; i < WBINS; i += NT) {
            uint32_t c = h[i];
            if (c) {
                atomicAdd(&gh[hw.base + i], c);
                h[i] = 0;
            }
        }
        // The histogram updates are device-scope atomics, performed where every CU sees
        // them; a thread only has to wait until its own have been acknowledged before the
        // workgroup is counted as arrived.  The workgroup that arrives last drops what it may
        // hold of the histogram in its caches and selects.
        wait_own_memory_ops();
        __syncthreads();
        if (tid == 0) s_last = atomicAdd(&ts.arrive_d[l], 1u) == gridDim.x - 1;
        __syncthreads();
        if (s_last) {  // uniform
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (tid == 0) ts.arrive_d[l] = 0;  // for the next call
            select_dense<DTYPE, NT>(l, sd, hist, sel, ts, s_sel);
        }
        __syncthreads();
    }
}

// fp32, dense route: histogram of the low 16 key bits of the entries in the threshold bin.
__global__ void __launch_bounds__(256)
hist2_kernel(const char *__restrict__ grad, const uint32_t *__restrict__ table,
             const SelDev *__restrict__ sel, uint32_t *__restrict__ hist2)
{
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    if (!any_dense_route(segs, sel, L)) return;
    const uint32_t tid = threadIdx.x;
    for (uint32_t l = 0; l < L; ++l) {
        const SegDev sd = segs[l];
        if (!on_dense_route(sd, sel, l) || !sel[l].need2) continue;
        const uint32_t bin1 = sel[l].bin1;
        uint32_t *gh = hist2 + uint64_t(l) * kBins2;
        const char *base = grad + sd.offset * 4;
        if (sd.flags & kSegAligned) {
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

// fp32, candidate route: the same histogram from the spilled candidates.
__global__ void __launch_bounds__(256)
hist2c_kernel(const uint32_t *__restrict__ table, const SelDev *__restrict__ sel,
              const uint32_t *__restrict__ cand, const uint2 *__restrict__ chunk_info,
              uint32_t n_slots_total, uint32_t CAP, uint32_t *__restrict__ hist2)
{
    constexpr uint32_t CHUNK = 64 * 4 * kCandRows;
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = gridDim.x * 4;
    for (uint32_t l = 0; l < L; ++l) {
        const SegDev sd = segs[l];
        if (sd.k == 0 || sd.n == 0 || on_dense_route(sd, sel, l) || !sel[l].need2) continue;
        const uint32_t bin1 = sel[l].bin1;
        uint32_t *gh = hist2 + uint64_t(l) * kBins2;
        const uint32_t n_chunks = (sd.n + CHUNK - 1) / CHUNK;
        for (uint32_t ch = wave; ch < n_chunks; ch += n_waves) {
            const uint32_t g = sd.sc_start * kCandChunksPerSuper + ch;
            const uint2 info = chunk_info[g];  // count, first slot
            const uint32_t c = min(info.x, CAP);
            const uint32_t first = min(info.y, n_slots_total - CAP);
            for (uint32_t i = lane; i < c; i += 64) {
                const uint32_t key = cand[first + i] & 0x7FFFFFFFu;
                if ((key >> 16) == bin1) atomicAdd(&gh[key & 0xFFFFu], 1u);
            }
        }
    }
}

__global__ void __launch_bounds__(kHistThreads)
select2_kernel(uint32_t *table, const uint32_t *__restrict__ hist2, SelDev *__restrict__ sel)
{
    __shared__ uint32_t smem[32];
    const uint32_t l = blockIdx.x;
    const SegDev sd = reinterpret_cast<const SegDev *>(table + 8)[l];
    if (sd.k == 0 || sd.n == 0) return;
    SelDev r = sel[l];
    if (!r.need2) return;
    uint32_t bin, above, at, total;
    bool found =
        select_bins<64>(hist2 + uint64_t(l) * kBins2, sd.k - r.G1, &bin, &above, &at, &total, smem);
    if (threadIdx.x != 0) return;
    if (!found) {  // cannot happen when both histograms saw the same data
        bin = 0;
        above = total;
        atomicOr(&table_state(table, table[0]).glob[0], TAGC_FLAG_OVERFLOW);
    }
    r.T = (r.bin1 << 16) | bin;
    r.G = r.G1 + above;
    r.quota = sd.k - r.G;
    r.cnt = sd.k;
    r.need2 = 0;
    sel[l] = r;
}

// ---------------------------------------------------------- ordered output

// Ordered output (the candidate route's super-chunks, the dense route's tiles) takes two
// launches and no waiting.  `count` leaves, per item, count(key > T) << 31 | count(key == T);
// `place` starts when all of them are there: every item adds up the counts of the earlier
// items of its segment by itself (a few hundred to a few thousand words from the L2) and puts
// its survivors where they belong.  No workgroup ever depends on another one's progress, so
// neither the order in which the device starts them nor other kernels in flight matter.

// last l with start(l) <= t, start() read through `field` (tile_start or sc_start)
template <typename F>
__device__ inline uint32_t segment_of(uint32_t L, uint32_t t, F start)
{
    uint32_t lo = 0, hi = L;
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (start(mid) <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// pairs segment i emits, as the selection left it (segments that keep nothing have none)
__device__ inline uint32_t segment_count(const SegDev &sd, const SelDev *sel, uint32_t i)
{
    return sd.k == 0 || sd.n == 0 ? 0u : sel[i].cnt;
}

// The rank's count words, from the selections and what the call's kernels accumulated in
// the table (which goes back to zero); by one workgroup of the last kernel.
__device__ inline void write_rank_counts(uint32_t *table, const SelDev *sel, uint32_t *cnt,
                                         uint32_t *smem /* >= 8 */)
{
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    uint32_t total = 0;
    for (uint32_t l = threadIdx.x; l < L; l += kEmitThreads) {
        const uint32_t c = segment_count(segs[l], sel, l);
        cnt[TAGC_CNT_SEG0 + l] = c;
        total += c;
    }
    total = block_sum<uint32_t, kEmitThreads / 64>(total, smem);
    if (threadIdx.x == 0) {
        const TableState ts = table_state(table, L);
        cnt[TAGC_CNT_TOTAL] = total;
        cnt[TAGC_CNT_FLAGS] = ts.glob[0];
        cnt[TAGC_CNT_NONFINITE] = ts.glob[1];
        cnt[TAGC_CNT_DENSE] = ts.glob[2];
        cnt[TAGC_CNT_RESERVED] = 0;
        ts.glob[0] = ts.glob[1] = ts.glob[2] = 0;
    }
}

// ------------------------------------------------------------------- emit

// Candidate route, count and place.  A workgroup handles kEmitItems adjacent super-chunks (32
// chunks each), two waves per super-chunk: 4 threads per chunk share the chunk's slots
// evenly, in order, and classify them against the exact threshold.  `count` (PLACE = false)
// stops there and stores the item's totals.  `place` classifies again, scans over the item's
// threads, adds up the earlier super-chunks of the segment and places the survivors in
// ascending c-index.  A super-chunk's Index words are assembled in LDS and written whole,
// zeros included.
//
// Every step is latency-bound (a dependent memory access costs 1-3 us under load), so the
// kernels are built to need few of them in a row and to be resident all at once (one item's
// state per thread keeps the register count low enough for that).  Everything whose
// address follows from the workgroup number alone is requested at once: the chunk counts,
// and -- lane i taking segment i -- the whole segment and selection tables, from which the
// item's segment, its threshold and the pair offset of the segment come by ballot,
// readlane and a wave sum (tables of more than 64 segments take a slower path).
//
// An item's survivors are consecutive in the output.  Stored entry by entry, each wave
// instruction would touch 64 different cache lines (measured: 60 % of the kernel's time);
// so the first kEmitStage of them are placed in LDS and leave as contiguous stores, and
// only what exceeds that (items keeping more than about 2 %) is stored directly.
constexpr uint32_t kEmitStage = 800;  // survivors of an item that go through LDS
static_assert(kEmitThreads == 128 * kEmitItems, "two waves per item");

template <int DTYPE, bool PLACE>
__device__ __forceinline__ void emit_body(uint32_t bid, uint32_t nb,
                                 const uint32_t *__restrict__ table,
                                 const SelDev *__restrict__ sel,
            const uint32_t *__restrict__ cand, const uint2 *__restrict__ chunk_info,
            uint64_t n_slots_total, uint32_t CAP, uint64_t *sc_cnt,
            uint32_t *__restrict__ idx_out, float *__restrict__ val_out,
            uint32_t *__restrict__ bitmap)
{
    constexpr uint32_t VEC = DTYPE == kBF16 ? 8 : 4;
    constexpr uint32_t CHUNK = 64 * VEC * kCandRows;
    constexpr uint32_t SC_ELEMS = CHUNK * kCandChunksPerSuper;
    constexpr uint32_t SC_WORDS = SC_ELEMS / 32;
    constexpr int NI = kEmitItems;
    __shared__ uint32_t bits[PLACE ? NI : 1][PLACE ? SC_WORDS : 1];
    // staged survivor: value bits and position in the super-chunk (16 bits); bf16 packs
    // both in one word, like a candidate slot
    __shared__ uint32_t st_a[PLACE ? NI : 1][PLACE ? kEmitStage : 1];
    __shared__ uint16_t st_b[PLACE ? NI : 1][PLACE && DTYPE == kF32 ? kEmitStage : 2];
    static_assert(SC_ELEMS <= 65536, "a position in the super-chunk fits 16 bits");
    __shared__ uint32_t s_gt[2 * NI], s_eq[2 * NI];
    __shared__ uint64_t s_sum[2 * NI];
    const uint32_t L = table[0], total_sc = table[4];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t k = wave >> 1;  // this wave's item within the workgroup
    const uint32_t tt = tid & 127;
    const uint32_t ch_in_sc = tt >> 2, part = tt & 3;

    for (uint32_t base = bid * NI; base < total_sc; base += nb * NI) {
        // ---- requests that depend on nothing but the item number
        const uint32_t sc = base + k;
        bool live = sc < total_sc;
        const uint32_t scc = live ? sc : 0u;
        const uint32_t g = scc * kCandChunksPerSuper + ch_in_sc;  // global chunk number
        // count and first slot (only meaningful for a chunk the scan has seen)
        const uint2 cinfo = chunk_info[g];
        const uint32_t craw = cinfo.x;
        // (the bound keeps the reads inside `cand` whatever an unseen chunk's record holds)
        const uint32_t *sp = cand + (min(cinfo.y, uint32_t(n_slots_total) - CAP) & ~3u);
        // segment i's table rows in lane i
        uint32_t t_start = 0xFFFFFFFFu, t_n = 0, t_coff = 0, t_T = 0, t_quota = 0, t_cnt = 0,
                 t_route = 0;
        if (L <= 64 && lane < L) {
            static_assert(sizeof(SegDev) == 32 && sizeof(SelDev) == 32, "two uint4 per row");
            const uint4 *s4 = reinterpret_cast<const uint4 *>(segs + lane);
            const uint4 *e4 = reinterpret_cast<const uint4 *>(sel + lane);
            const uint4 sa = s4[0], sb = s4[1], ea = e4[0], eb = e4[1];
            t_n = sa.z; t_coff = sa.w; t_start = sb.w;                 // n, c_off, sc_start
            if (sb.x != 0 && sa.z != 0) {   // k, n: a segment that keeps nothing has no selection
                t_T = ea.x; t_quota = ea.y; t_cnt = ea.w; t_route = eb.w;  // T, quota, cnt, route
            }
        }
        if (PLACE)
            for (uint32_t i = tt; i < SC_WORDS; i += 128) bits[k][i] = 0;

        // ---- segment, threshold, pair offset of the segment (all wave-uniform)
        uint32_t l, c_off, n_seg, sc_first, T, quota, seg_base, se_cnt, se_route;
        if (L <= 64) {
            const uint64_t le = __ballot(t_start <= scc);  // a prefix of the lanes
            l = uint32_t(__popcll(le)) - 1u;               // segment 0 starts at 0
            n_seg = __builtin_amdgcn_readlane(t_n, l);
            c_off = __builtin_amdgcn_readlane(t_coff, l);
            sc_first = __builtin_amdgcn_readlane(t_start, l);
            T = __builtin_amdgcn_readlane(t_T, l);
            quota = __builtin_amdgcn_readlane(t_quota, l);
            se_cnt = __builtin_amdgcn_readlane(t_cnt, l);
            se_route = __builtin_amdgcn_readlane(t_route, l);
            seg_base = wave_sum<uint32_t>(lane < l ? t_cnt : 0u);
        } else {
            l = segment_of(L, scc, [&](uint32_t i) { return segs[i].sc_start; });
            const SegDev sd = segs[l];
            SelDev se{};
            if (sd.k != 0 && sd.n != 0) se = sel[l];
            n_seg = sd.n; c_off = sd.c_off; sc_first = sd.sc_start;
            T = se.T; quota = se.quota; se_cnt = se.cnt; se_route = se.route;
            uint32_t sum = 0;
            for (uint32_t i = lane; i < l; i += 64) sum += segment_count(segs[i], sel, i);
            seg_base = wave_sum<uint32_t>(sum);
        }
        live = live && !se_route;  // the dense route writes re-routed segments
        const uint32_t sc_rel0 = (scc - sc_first) * SC_ELEMS;
        const bool in_seg = live && se_cnt != 0 && sc_rel0 + ch_in_sc * CHUNK < n_seg;
        const uint32_t ccnt = in_seg ? min(craw, CAP) : 0u;
        // the chunk's slots in four equal runs of whole 16-byte groups, one per thread
        const uint32_t run = ((ccnt + 3) / 4 + 3) & ~3u;
        const uint32_t s0 = min(part * run, ccnt), s1 = min(s0 + run, ccnt);
        // The first two 16-byte groups of the run (all of it unless the chunk holds more
        // than 32 candidates) are requested together and kept for both passes; a longer
        // run reads the rest group by group.
        constexpr uint32_t QN = 2;
        uint4 q[QN], qp[QN];
#pragma unroll
        for (uint32_t j = 0; j < QN; ++j) {
            q[j] = qp[j] = make_uint4(0, 0, 0, 0);
            if (s0 + 4 * j < s1) {
                q[j] = *reinterpret_cast<const uint4 *>(sp + s0 + 4 * j);
                if (DTYPE == kF32)
                    qp[j] = *reinterpret_cast<const uint4 *>(sp + n_slots_total + s0 + 4 * j);
            }
        }
        // fn(value bits, position in chunk) for every slot of this thread
        auto for_slots = [&](auto &&fn) {
#pragma unroll
            for (uint32_t j = 0; j < QN; ++j) {
                const uint32_t v[4] = {q[j].x, q[j].y, q[j].z, q[j].w};
                const uint32_t rp[4] = {qp[j].x, qp[j].y, qp[j].z, qp[j].w};
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i) {
                    if (s0 + 4 * j + i >= s1) continue;
                    if (DTYPE == kBF16) fn(v[i] & 0xFFFF0000u, v[i] & 0xFFFFu);
                    else fn(v[i], rp[i]);
                }
            }
            for (uint32_t s4 = s0 + 4 * QN; s4 < s1; s4 += 4) {
                const uint4 a = *reinterpret_cast<const uint4 *>(sp + s4);
                uint4 b = make_uint4(0, 0, 0, 0);
                if (DTYPE == kF32) b = *reinterpret_cast<const uint4 *>(sp + n_slots_total + s4);
                const uint32_t v[4] = {a.x, a.y, a.z, a.w};
                const uint32_t rp[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i) {
                    if (s4 + i >= s1) continue;
                    if (DTYPE == kBF16) fn(v[i] & 0xFFFF0000u, v[i] & 0xFFFFu);
                    else fn(v[i], rp[i]);
                }
            }
        };
        // ---- pass 1: count this thread's slots above / at the threshold
        uint32_t n_gt = 0, n_eq = 0;
        for_slots([&](uint32_t vbits, uint32_t) {
            const uint32_t key = vbits & 0x7FFFFFFFu;
            n_gt += key > T;
            n_eq += (key == T) && quota;
        });
        // ---- order inside the item (its 128 threads are in position order)
        const uint32_t inc_gt = wave_incl_scan<uint32_t>(n_gt);
        const uint32_t inc_eq = wave_incl_scan<uint32_t>(n_eq);
        if (lane == 63) {
            s_gt[wave] = inc_gt;
            s_eq[wave] = inc_eq;
        }
        __syncthreads();
        const uint32_t lo_gt = s_gt[2 * k], lo_eq = s_eq[2 * k];
        const uint32_t it_gt = lo_gt + s_gt[2 * k + 1], it_eq = lo_eq + s_eq[2 * k + 1];
        if (!PLACE) {
            if (sc < total_sc && tt == 0) sc_cnt[sc] = (uint64_t(it_gt) << 31) | uint64_t(it_eq);
            __syncthreads();  // s_gt / s_eq are rewritten by the next iteration
            continue;
        }
        uint32_t gb = inc_gt - n_gt + ((wave & 1u) ? lo_gt : 0u);
        uint32_t eb = inc_eq - n_eq + ((wave & 1u) ? lo_eq : 0u);
        // ---- prefix over the segment's earlier super-chunks, whose counts are all there
        uint64_t sum = 0;
        if (live)
            for (uint32_t j = sc_first + tt; j < sc; j += 128) sum += sc_cnt[j];
        sum = wave_sum<uint64_t>(sum);
        if (lane == 0) s_sum[wave] = sum;
        __syncthreads();  // also orders the clearing of `bits` before the ORs below
        sum = s_sum[2 * k] + s_sum[2 * k + 1];
        // output position (within the segment) of the item's first survivor, and how many
        // survivors the item has: entries above T all survive, ties while the quota lasts
        const uint32_t pre_gt = uint32_t(sum >> 31), pre_eq = uint32_t(sum & 0x7FFFFFFFu);
        const uint32_t item_pos = pre_gt + min(pre_eq, quota);
        const uint32_t item_n = pre_gt + it_gt + min(pre_eq + it_eq, quota) - item_pos;
        gb += pre_gt;
        eb += pre_eq;
        // ---- pass 2: place the survivors
        if (n_gt | n_eq) {
            for_slots([&](uint32_t vbits, uint32_t rel) {
                const uint32_t key = vbits & 0x7FFFFFFFu;
                uint32_t pos;
                bool keep;
                if (key > T) {
                    pos = gb + min(eb, quota);
                    keep = true;
                    ++gb;
                } else if (key == T && quota) {
                    pos = gb + eb;
                    keep = eb < quota;
                    ++eb;
                } else {
                    return;
                }
                if (keep) {
                    const uint32_t rel_sc = ch_in_sc * CHUNK + rel;
                    const uint32_t ci = c_off + sc_rel0 + rel_sc;
                    const uint32_t p = pos - item_pos;
                    if (p < kEmitStage) {
                        if (DTYPE == kBF16) {
                            st_a[k][p] = vbits | rel_sc;
                        } else {
                            st_a[k][p] = vbits;
                            st_b[k][DTYPE == kF32 ? p : 0] = uint16_t(rel_sc);
                        }
                    } else {
                        idx_out[seg_base + pos] = ci;
                        val_out[seg_base + pos] = __uint_as_float(vbits);
                    }
                    atomicOr(&bits[k][rel_sc >> 5], 1u << (rel_sc & 31));
                }
            });
        }
        __syncthreads();
        if (live) {
            const uint32_t n_st = min(item_n, kEmitStage);
            for (uint32_t i = tt; i < n_st; i += 128) {
                const uint32_t a = st_a[k][i];
                const uint32_t rel_sc = DTYPE == kBF16 ? (a & 0xFFFFu) : st_b[k][DTYPE == kF32 ? i : 0];
                idx_out[seg_base + item_pos + i] = c_off + sc_rel0 + rel_sc;
                val_out[seg_base + item_pos + i] =
                    __uint_as_float(DTYPE == kBF16 ? (a & 0xFFFF0000u) : a);
            }
            const uint32_t w0 = (c_off + sc_rel0) >> 5;
            for (uint32_t i = tt; i < SC_WORDS; i += 128)
                if (sc_rel0 + i * 32 < n_seg) bitmap[w0 + i] = bits[k][i];
        }
        __syncthreads();  // LDS is reused by the next iteration
    }
}

// ------------------------------------------------- emit, a wave per super-chunk

// emit_body gives a chunk's slots to four threads, which suits the few dozen candidates a
// chunk holds when one entry in a hundred is kept, and stages an item's survivors in LDS.
// Where a tenth or a fifth is kept (the 4x and 2x regimes of Table 1) a chunk holds
// hundreds; and the LDS (23 KiB per workgroup in place) keeps all but two of its workgroups
// off a compute unit on which another bucket's scan is running, which is how large buckets
// are usually processed.  Here a wave takes a whole super-chunk
// and reads its chunks' slots 64 at a time, in position order, BATCH such reads in
// flight.  The survivors among the 64 slots of one read are neighbours in the output, so
// they are stored as they are found; the Index words of a chunk are collected in LDS and
// leave when its last slots are through.  Same inputs, same outputs, same counts per
// super-chunk as emit_body.
template <int DTYPE, bool PLACE, uint32_t BATCH>
__device__ __forceinline__ void emit_wide_body(uint32_t bid, uint32_t nb,
                                 const uint32_t *__restrict__ table,
                                 const SelDev *__restrict__ sel,
            const uint32_t *__restrict__ cand, const uint2 *__restrict__ chunk_info,
            uint64_t n_slots_total, uint32_t CAP, uint64_t *sc_cnt,
            uint32_t *__restrict__ idx_out, float *__restrict__ val_out,
            uint32_t *__restrict__ bitmap)
{
    constexpr uint32_t VEC = DTYPE == kBF16 ? 8 : 4;
    constexpr uint32_t CHUNK = 64 * VEC * kCandRows;
    constexpr uint32_t NCH = kCandChunksPerSuper;
    constexpr uint32_t SC_ELEMS = CHUNK * NCH;
    constexpr uint32_t CH_WORDS = CHUNK / 32;
    constexpr uint32_t NWV = kEmitThreads / 64;
    static_assert(NCH <= 64 && CH_WORDS <= 64, "a lane per chunk, a lane per Index word of a chunk");
    __shared__ uint32_t wbits[PLACE ? NWV : 1][PLACE ? CH_WORDS : 1];  // a wave's current chunk
    const uint32_t L = table[0], total_sc = table[4];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t lanes_below = (1ull << lane) - 1ull;

    // segment i's table rows in lane i
    uint32_t t_start = 0xFFFFFFFFu, t_n = 0, t_coff = 0, t_T = 0, t_quota = 0, t_cnt = 0,
             t_route = 0;
    if (L <= 64 && lane < L) {
        const uint4 *s4 = reinterpret_cast<const uint4 *>(segs + lane);
        const uint4 *e4 = reinterpret_cast<const uint4 *>(sel + lane);
        const uint4 sa = s4[0], sb = s4[1], ea = e4[0], eb4 = e4[1];
        t_n = sa.z; t_coff = sa.w; t_start = sb.w;                 // n, c_off, sc_start
        if (sb.x != 0 && sa.z != 0) {   // k, n: a segment that keeps nothing has no selection
            t_T = ea.x; t_quota = ea.y; t_cnt = ea.w; t_route = eb4.w;  // T, quota, cnt, route
        }
    }
    if (PLACE && lane < CH_WORDS) wbits[wave][lane] = 0;  // (no other wave touches this row)

    for (uint32_t sc = bid * NWV + wave; sc < total_sc; sc += nb * NWV) {  // wave-uniform
        // ---- segment, threshold, pair offset of the segment
        uint32_t l, c_off, n_seg, sc_first, T, quota, seg_base, se_cnt, se_route;
        if (L <= 64) {
            const uint64_t le = __ballot(t_start <= sc);  // a prefix of the lanes
            l = uint32_t(__popcll(le)) - 1u;              // segment 0 starts at 0
            n_seg = __builtin_amdgcn_readlane(t_n, l);
            c_off = __builtin_amdgcn_readlane(t_coff, l);
            sc_first = __builtin_amdgcn_readlane(t_start, l);
            T = __builtin_amdgcn_readlane(t_T, l);
            quota = __builtin_amdgcn_readlane(t_quota, l);
            se_cnt = __builtin_amdgcn_readlane(t_cnt, l);
            se_route = __builtin_amdgcn_readlane(t_route, l);
            seg_base = wave_sum<uint32_t>(lane < l ? t_cnt : 0u);
        } else {
            l = segment_of(L, sc, [&](uint32_t i) { return segs[i].sc_start; });
            const SegDev sd = segs[l];
            SelDev se{};
            if (sd.k != 0 && sd.n != 0) se = sel[l];
            n_seg = sd.n; c_off = sd.c_off; sc_first = sd.sc_start;
            T = se.T; quota = se.quota; se_cnt = se.cnt; se_route = se.route;
            uint32_t sum = 0;
            for (uint32_t i = lane; i < l; i += 64) sum += segment_count(segs[i], sel, i);
            seg_base = wave_sum<uint32_t>(sum);
        }
        const bool live = !se_route;  // the dense route writes re-routed segments
        const uint32_t sc_rel0 = (sc - sc_first) * SC_ELEMS;

        // ---- chunk `lane` of the super-chunk: its candidates and where their slots are
        // (the bound keeps the reads inside `cand` whatever the record holds)
        bool inseg_l = false;
        uint32_t cnt_l = 0, first_l = 0;
        if (lane < NCH) {
            inseg_l = live && sc_rel0 + lane * CHUNK < n_seg;
            if (inseg_l && se_cnt != 0) {
                const uint2 info = chunk_info[sc * NCH + lane];
                cnt_l = min(info.x, CAP);
                first_l = min(info.y, uint32_t(n_slots_total) - CAP);
            }
        }
        // Reads of 64 slots ("groups"), numbered through the super-chunk.  Where no chunk
        // needs a second read (a few dozen candidates per chunk) group g is simply chunk g.
        const uint32_t ngr_l = (cnt_l + 63u) >> 6;
        const uint32_t gend_l = wave_incl_scan<uint32_t>(ngr_l);  // (lanes from NCH on: the total)
        const bool one_each = __ballot(ngr_l > 1u) == 0;
        const uint32_t n_groups = one_each ? NCH : __builtin_amdgcn_readlane(gend_l, 63);
        const uint32_t ins_l = inseg_l ? 1u : 0u;
        // where group g lies (all wave-uniform): chunk, first slot, slots of the chunk
        auto locate = [&](uint32_t g, uint32_t &ch, uint32_t &c, uint32_t &s0, uint32_t &first) {
            if (one_each) {
                ch = g;
                s0 = 0;
            } else {
                ch = uint32_t(__popcll(__ballot(gend_l <= g)));  // chunks that end before g
                const uint32_t gbeg = __builtin_amdgcn_readlane(gend_l, ch) -
                                      __builtin_amdgcn_readlane(ngr_l, ch);
                s0 = (g - gbeg) * 64;
            }
            c = __builtin_amdgcn_readlane(cnt_l, ch);
            first = __builtin_amdgcn_readlane(first_l, ch);
        };
        uint32_t v[BATCH], vp[BATCH];
        auto request = [&](uint32_t b0) {
#pragma unroll
            for (uint32_t j = 0; j < BATCH; ++j) {
                v[j] = vp[j] = 0;
                if (b0 + j < n_groups) {
                    uint32_t ch, c, s0, first;
                    locate(b0 + j, ch, c, s0, first);
                    if (s0 + lane < c) {
                        v[j] = cand[first + s0 + lane];
                        if (DTYPE == kF32) vp[j] = cand[n_slots_total + first + s0 + lane];
                    }
                }
            }
        };
        request(0);  // (on their way while the prefix below is added up)

        uint32_t gb = 0, eb = 0;  // entries above / at the threshold before the current slot
        if (PLACE) {
            // prefix over the segment's earlier super-chunks, whose counts are all there
            uint64_t sum = 0;
            if (live)
                for (uint32_t j = sc_first + lane; j < sc; j += 64) sum += sc_cnt[j];
            sum = wave_sum<uint64_t>(sum);
            gb = uint32_t(sum >> 31);
            eb = uint32_t(sum & 0x7FFFFFFFu);
            // chunks of the segment without a candidate have no group of their own unless
            // group = chunk: their Index words are zero
            if (!one_each) {
                for (uint64_t em = __ballot(inseg_l && cnt_l == 0); em; em &= em - 1) {
                    const uint32_t ch = uint32_t(__builtin_ctzll(em));
                    const uint32_t rel0 = sc_rel0 + ch * CHUNK + lane * 32;
                    if (lane < CH_WORDS && rel0 < n_seg) bitmap[(c_off + rel0) >> 5] = 0;
                }
            }
        }

        for (uint32_t b0 = 0; b0 < n_groups;) {
#pragma unroll
            for (uint32_t j = 0; j < BATCH; ++j) {
                if (b0 + j >= n_groups) continue;
                uint32_t ch, c, s0, first;
                locate(b0 + j, ch, c, s0, first);
                const bool valid = s0 + lane < c;
                const uint32_t vbits = DTYPE == kBF16 ? (v[j] & 0xFFFF0000u) : v[j];
                const uint32_t rel = (DTYPE == kBF16 ? (v[j] & 0xFFFFu) : vp[j]) & (CHUNK - 1u);
                const uint32_t key = vbits & 0x7FFFFFFFu;
                const bool is_gt = valid && key > T;
                const bool is_eq = valid && key == T && quota != 0;
                const uint64_t bgt = __ballot(is_gt), beq = __ballot(is_eq);
                if (PLACE) {
                    const uint32_t my_gb = gb + uint32_t(__popcll(bgt & lanes_below));
                    const uint32_t my_eb = eb + uint32_t(__popcll(beq & lanes_below));
                    // entries above T all survive, ties while the quota lasts
                    const bool keep = is_gt || (is_eq && my_eb < quota);
                    if (keep) {
                        const uint32_t pos = is_gt ? my_gb + min(my_eb, quota) : my_gb + my_eb;
                        idx_out[seg_base + pos] = c_off + sc_rel0 + ch * CHUNK + rel;
                        val_out[seg_base + pos] = __uint_as_float(vbits);
                        atomicOr(&wbits[wave][rel >> 5], 1u << (rel & 31));
                    }
                    // the chunk's last slots: its Index words leave
                    if (s0 + 64 >= c && __builtin_amdgcn_readlane(ins_l, ch)) {
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        if (lane < CH_WORDS) {
                            const uint32_t w = wbits[wave][lane];
                            wbits[wave][lane] = 0;
                            const uint32_t rel0 = sc_rel0 + ch * CHUNK + lane * 32;
                            if (rel0 < n_seg) bitmap[(c_off + rel0) >> 5] = w;
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
                }
                gb += uint32_t(__popcll(bgt));
                eb += uint32_t(__popcll(beq));
            }
            b0 += BATCH;
            if (b0 < n_groups) request(b0);
        }
        if (!PLACE && lane == 0) sc_cnt[sc] = (uint64_t(gb) << 31) | uint64_t(eb);
    }
}

// ---------------------------------------------------------------- compact

// Dense route, count and place, over the gradient itself: one tile of kCompactThreads x ROWS
// 16-byte vectors per workgroup and turn.  Also writes the (all-zero) Index words of the
// segments that keep nothing.
template <int DTYPE, uint32_t ROWS, bool PLACE>
__device__ __forceinline__ void compact_body(uint32_t bid, uint32_t nb, const char *grad,
                                    const uint32_t *__restrict__ table,
               const SelDev *__restrict__ sel, uint64_t *tile_cnt, uint64_t *group_cnt,
               uint32_t *__restrict__ idx_out,
               float *__restrict__ val_out, uint32_t *__restrict__ bitmap)
{
    constexpr uint32_t EB = DTYPE == kBF16 ? 2 : 4;
    constexpr uint32_t VEC = 16 / EB;
    constexpr uint32_t ROW_ELEMS = kCompactThreads * VEC;
    constexpr uint32_t TILE = ROW_ELEMS * ROWS;
    constexpr uint32_t LPW = 32 / VEC;  // lanes that share one Index word
    __shared__ uint64_t s_scan[2 * (kCompactThreads / 64)];
    __shared__ uint64_t s_excl;
    __shared__ uint32_t s_base;

    const uint32_t L = table[0], total_tiles = table[1];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    // anything to do at all?  (uniform: every thread reads the same words)
    bool any = false;
    for (uint32_t l = 0; l < L; ++l) {
        const SegDev sd = segs[l];
        any |= on_dense_route(sd, sel, l) || (PLACE && sd.n != 0 && sd.k == 0);
    }
    if (!any) return;
    const uint32_t tid = threadIdx.x;

    for (uint32_t t = bid; t < total_tiles; t += nb) {
        const uint32_t l = segment_of(L, t, [&](uint32_t i) { return segs[i].tile_start; });
        const SegDev sd = segs[l];
        const bool dense = on_dense_route(sd, sel, l);
        // (the candidate route writes the other segments that keep something; a segment that
        // keeps nothing only needs its Index words, which place writes as zeros)
        if (!dense && !(PLACE && sd.n != 0 && sd.k == 0)) continue;  // uniform
        SelDev se{};
        if (dense) se = sel[l];
        const uint32_t base_rel = (t - sd.tile_start) * TILE;
        if (base_rel >= sd.n) continue;  // (tile_start of several empty segments coincides)
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
                if ((sd.flags & kSegAligned) && rel + VEC <= sd.n) {
                    const uint4 q =
                        ld_stream(reinterpret_cast<const uint4 *>(base + uint64_t(rel) * EB));
                    w[r][0] = q.x; w[r][1] = q.y; w[r][2] = q.z; w[r][3] = q.w;
                } else {
                    const uint32_t cntv = min(VEC, sd.n - rel);
#pragma unroll
                    for (uint32_t e = 0; e < VEC; ++e) {
                        if (e >= cntv) continue;
                        const uint32_t b = load_elem_bits(base, uint64_t(rel) + e, DTYPE);
                        if (DTYPE == kBF16) w[r][e >> 1] |= (b >> 16) << (16 * (e & 1));
                        else w[r][e] = b;
                    }
                }
            }
            // ---- classify.  Elements past the end were loaded as 0 and are never kept.
#pragma unroll
            for (uint32_t r = 0; r < ROWS; ++r) {
#pragma unroll
                for (uint32_t e = 0; e < VEC; ++e) {
                    const uint32_t key = vec_elem_bits<DTYPE>(w[r], e) & 0x7FFFFFFFu;
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
        if (!PLACE) {
            // the tile's counts, and added to those of its group of kTileGroup tiles (groups
            // are cut from the bucket's tile numbers, whatever the segments)
            if (tid == 0) {
                const uint64_t v = (uint64_t(Gt) << 31) | Et;
                tile_cnt[t] = v;
                atomicAdd(reinterpret_cast<unsigned long long *>(&group_cnt[t / kTileGroup]), v);
            }
            continue;  // (block_excl_scan ends with a barrier: s_scan may be reused)
        }
        // ---- add up the counts of the segment's earlier tiles: whole groups that lie inside
        // the segment by their sums, the tiles before and after them one by one (a few
        // hundred words at most, from the L2); pair offset of the segment
        {
            uint64_t sum = 0;
            if (dense) {
                const uint32_t t0 = sd.tile_start;
                const uint32_t g0 = (t0 + kTileGroup - 1) / kTileGroup, g1 = t / kTileGroup;
                if (g0 < g1) {
                    for (uint32_t j = t0 + tid; j < g0 * kTileGroup; j += kCompactThreads) sum += tile_cnt[j];
                    for (uint32_t j = g0 + tid; j < g1; j += kCompactThreads) sum += group_cnt[j];
                    for (uint32_t j = g1 * kTileGroup + tid; j < t; j += kCompactThreads) sum += tile_cnt[j];
                } else {
                    for (uint32_t j = t0 + tid; j < t; j += kCompactThreads) sum += tile_cnt[j];
                }
            }
            sum = block_sum<uint64_t, kCompactThreads / 64>(sum, s_scan);
            uint32_t sb = 0;
            if (tid < 64) {
                for (uint32_t i = tid; i < l; i += 64) sb += segment_count(segs[i], sel, i);
                sb = wave_sum<uint32_t>(sb);
            }
            if (tid == 0) {
                s_excl = sum;
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
                    uint32_t bits = 0;
#pragma unroll
                    for (uint32_t j = 0; j < VEC; ++j)
                        if (j == e) bits = vec_elem_bits<DTYPE>(w[r], j);
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

// --------------------------------------------------------- count and place

// The last two kernels of PHASE_INDEX.  In each, the first `n_emit` workgroups work on the
// candidate-route segments and the rest on the dense-route ones (pairs and Index words of
// different segments): one launch instead of two, and when a bucket has no dense-route work
// that part costs nothing, not even an empty kernel's turn-around.
static_assert(kEmitThreads == kCompactThreads, "one launch for both parts");

template <int DTYPE, uint32_t COMPACT_ROWS, bool WIDE>
__global__ void __launch_bounds__(kEmitThreads)
count_kernel(uint32_t n_emit, const char *grad, const uint32_t *__restrict__ table,
             const SelDev *__restrict__ sel, const uint32_t *__restrict__ cand,
             const uint2 *__restrict__ chunk_info, uint64_t n_slots_total, uint32_t CAP,
             uint64_t *sc_cnt, uint64_t *tile_cnt, uint64_t *group_cnt)
{
    if (blockIdx.x < n_emit) {
        if (WIDE)
            emit_wide_body<DTYPE, false, 32>(blockIdx.x, n_emit, table, sel, cand, chunk_info,
                                         n_slots_total, CAP, sc_cnt, nullptr, nullptr, nullptr);
        else
            emit_body<DTYPE, false>(blockIdx.x, n_emit, table, sel, cand, chunk_info,
                                    n_slots_total, CAP, sc_cnt, nullptr, nullptr, nullptr);
    } else
        compact_body<DTYPE, COMPACT_ROWS, false>(blockIdx.x - n_emit, gridDim.x - n_emit, grad,
                                                 table, sel, tile_cnt, group_cnt, nullptr, nullptr,
                                                 nullptr);
}

template <int DTYPE, uint32_t COMPACT_ROWS, bool WIDE>
__global__ void __launch_bounds__(kEmitThreads)
    __attribute__((amdgpu_waves_per_eu(COMPACT_ROWS == 2 ? 7 : 6, 8)))
place_kernel(uint32_t n_emit, const char *grad, uint32_t *table,
             const SelDev *__restrict__ sel, const uint32_t *__restrict__ cand,
             const uint2 *__restrict__ chunk_info, uint64_t n_slots_total, uint32_t CAP,
             uint64_t *sc_cnt, uint64_t *tile_cnt, uint64_t *group_cnt,
             uint32_t *__restrict__ idx_out, float *__restrict__ val_out,
             uint32_t *__restrict__ bitmap, uint32_t *cnt)
{
    if (blockIdx.x == gridDim.x - 1) {  // (any one workgroup: the last has the least to do)
        __shared__ uint32_t s_cnt[8];
        write_rank_counts(table, sel, cnt, s_cnt);
    }
    if (blockIdx.x < n_emit) {
        if (WIDE)
            emit_wide_body<DTYPE, true, 16>(blockIdx.x, n_emit, table, sel, cand, chunk_info,
                                        n_slots_total, CAP, sc_cnt, idx_out, val_out, bitmap);
        else
            emit_body<DTYPE, true>(blockIdx.x, n_emit, table, sel, cand, chunk_info,
                                   n_slots_total, CAP, sc_cnt, idx_out, val_out, bitmap);
    } else
        compact_body<DTYPE, COMPACT_ROWS, true>(blockIdx.x - n_emit, gridDim.x - n_emit, grad,
                                                table, sel, tile_cnt, group_cnt, idx_out, val_out,
                                                bitmap);
}

template <typename K>
int resident_blocks_per_cu(K kernel, int threads, size_t lds, int *cache)
{
    if (*cache == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, lds) != hipSuccess ||
            n <= 0)
            return 0;
        *cache = n;
    }
    return *cache;
}

template <typename K>
int allow_lds(K kernel, size_t lds, bool *done)
{
    if (*done) return TAGC_OK;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
        return TAGC_EHIP;
    *done = true;
    return TAGC_OK;
}

// Error feedback, on request: clears the entries of acc that the rank's Index names, after
// which acc is acc_next of Algorithm 1 as a plain array (for inspection or a checkpoint;
// the next PHASE_INDEX call does not need it and gives the same results either way).  One
// thread per 32 parameters of the c-index space; ~1 % of the entries get a store.
__global__ void __launch_bounds__(256)
feedback_apply_kernel(const uint32_t *__restrict__ table, const SentMap sent, uint32_t n_words,
                      char *acc, int dtype)
{
    const uint32_t w = blockIdx.x * 256 + threadIdx.x;
    if (w >= n_words) return;
    uint32_t bits;
    if (sent.wire4) {
        const uint4 q = *reinterpret_cast<const uint4 *>(sent.map + 4 * size_t(w));
        bits = nibbles_set(q.x) | (nibbles_set(q.y) << 8) | (nibbles_set(q.z) << 16) |
               (nibbles_set(q.w) << 24);
    } else {
        bits = sent.map[w];
    }
    if (!bits) return;
    const uint32_t L = table[0];
    const SegDev *segs = reinterpret_cast<const SegDev *>(table + 8);
    // a word of the Index lies inside one segment (c-offsets are multiples of 32); of several
    // segments starting at the same c-index only the last is not empty
    const uint32_t l = segment_of(L, w * 32, [&](uint32_t i) { return segs[i].c_off; });
    const SegDev sd = segs[l];
    char *ab = acc + sd.offset * (dtype == kBF16 ? 2 : 4);
    const uint32_t rel0 = w * 32 - sd.c_off;
    for (; bits; bits &= bits - 1) {
        const uint32_t rel = rel0 + __builtin_ctz(bits);
        if (rel < sd.n) store_elem(ab, rel, 0u, dtype);
    }
}

// 4-bit wire Index (section 2.2: the stable, four times bigger variant that an All-Reduce
// by addition can merge): one 0/1 counter per parameter, parameter j in bits 4*(j&7).. of
// word j>>3.  One thread per word of the 1-bit Index: 4 bytes in, one 16-byte store out.
__device__ __forceinline__ uint32_t spread8(uint32_t b)  // bit p of a byte -> bit 4p
{
    uint32_t x = (b | (b << 12)) & 0x000F000Fu;  // nibbles 0,1 -> 16-bit fields
    x = (x | (x << 6)) & 0x03030303u;            // 2 bits per byte
    x = (x | (x << 3)) & 0x11111111u;            // 1 bit per nibble
    return x;
}

__global__ void __launch_bounds__(256)
widen4_kernel(const uint32_t *__restrict__ map, uint32_t n_words, uint32_t *__restrict__ wire)
{
    const uint32_t w = blockIdx.x * 256 + threadIdx.x;
    if (w >= n_words) return;
    const uint32_t m = map[w];
    st_stream(reinterpret_cast<uint4 *>(wire + 4 * size_t(w)),
              make_uint4(spread8(m & 0xFFu), spread8((m >> 8) & 0xFFu),
                         spread8((m >> 16) & 0xFFu), spread8(m >> 24)));
}

template <int DTYPE>
int launch_sparsify_t(const tagc_plan_t *p, const void *grad, const tagc_rank_buffers *rk,
                      const tagc_shared_buffers *sh, hipStream_t s)
{
    const uint32_t L = uint32_t(p->table.size());
    // the table is the plan's device state as well (pre-thresholds, counters): written here
    uint32_t *table = static_cast<uint32_t *>(const_cast<void *>(sh->table));
    char *ws = static_cast<char *>(rk->workspace);
    uint32_t *hist1d = reinterpret_cast<uint32_t *>(ws + p->ws.hist1d);
    uint32_t *hist2 = reinterpret_cast<uint32_t *>(ws + p->ws.hist2);
    uint64_t *tile_cnt = reinterpret_cast<uint64_t *>(ws + p->ws.tile_cnt);
    uint64_t *group_cnt = reinterpret_cast<uint64_t *>(ws + p->ws.group_cnt);
    uint64_t *sc_cnt = reinterpret_cast<uint64_t *>(ws + p->ws.sc_cnt);
    SelDev *sel = reinterpret_cast<SelDev *>(ws + p->ws.sel);
    uint2 *chunk_info = reinterpret_cast<uint2 *>(ws + p->ws.chunk_info);
    uint32_t *cand = reinterpret_cast<uint32_t *>(ws + p->ws.cand);
    const uint64_t n_slots = uint64_t(p->total_sc) * kCandChunksPerSuper * p->cand_cap;
    const char *g = static_cast<const char *>(grad);
    // with 4-bit counters on the wire the 1-bit Index is built in the workspace and widened
    const bool wide = p->cfg.index_mode == TAGC_INDEX_ADD4;
    uint32_t *bitmap1 = wide ? reinterpret_cast<uint32_t *>(ws + p->ws.bitmap1) : rk->bitmap;
    // Error feedback: scan_spill (candidate route) and accumulate_kernel (all other segments)
    // turn acc into grad + acc; whoever reads the input after them reads it from acc.  Both
    // read acc through the Index this rank's previous call left in rk->bitmap (what was
    // sent reads as 0) before place / widen4 overwrite that Index with the new one.
    char *acc = static_cast<char *>(rk->acc);
    const char *src = acc ? acc : g;
    const SentMap sent{rk->bitmap, wide ? 1u : 0u};
    const int cus = device_cu_count();
    const size_t lds_hist = kBins1 * sizeof(uint32_t);
    static bool a_prepare = false, a_hist = false;
    static int occ_place[2][2] = {{0, 0}, {0, 0}};

    if (L == 0 || (p->total_sc == 0 && p->total_tiles == 0)) {
        // nothing is compressed (or every compressed segment is empty): only the counts
        // have to read zero
        ProfileScope ps("fill_zero", s);
        fill_zero_kernel<<<1, 256, 0, s>>>(reinterpret_cast<uint4 *>(ws), 0, rk->cnt,
                                           TAGC_CNT_SEG0 + L);
        return hip_ok(hipGetLastError());
    }
    if (allow_lds(prepare_kernel<DTYPE>, lds_hist, &a_prepare) ||
        allow_lds(hist1_kernel<DTYPE, kBins1, kHistThreads>, lds_hist, &a_hist))
        return TAGC_EHIP;
    if (acc && p->any_nonfast) {
        ProfileScope ps("accumulate", s);
        accumulate_kernel<DTYPE><<<cus * 4, 256, 0, s>>>(g, table, acc, sent);
    }
    // the dense route's histograms are cleared by the scan as it starts, or, where there is
    // no scan, by prepare; which also samples pre-thresholds on the first call after an upload
    const uint64_t zero_n16 = p->zero_bytes / 16;
    const bool sample = p->sample_pending.exchange(0, std::memory_order_relaxed) != 0;
    if (sample || !p->total_sc) {
        ProfileScope ps("prepare", s);
        const uint64_t n16 = p->total_sc ? 0 : zero_n16;
        const uint32_t fill_blocks = uint32_t(
            std::max<uint64_t>(1, std::min<uint64_t>((n16 + kHistThreads - 1) / kHistThreads, cus)));
        prepare_kernel<DTYPE><<<L + fill_blocks, kHistThreads, lds_hist, s>>>(
            g, acc, sent, table, reinterpret_cast<uint4 *>(ws), n16);
    }
    if (p->total_sc) {
        ProfileScope ps("scan_spill", s);
        scan_spill_kernel<DTYPE><<<cus * kSpillWgsPerCU, kSpillThreads, 0, s>>>(
            g, acc, sent, table, sel, cand, chunk_info, n_slots, p->cand_cap,
            reinterpret_cast<uint4 *>(ws), zero_n16);
    }
    {
        // leaves at once unless a segment is on the dense route (by plan, or because the
        // scan's selection sent it there)
        ProfileScope ps("hist1", s);
        if (p->static_dense)
            hist1_kernel<DTYPE, kBins1, kHistThreads><<<cus, kHistThreads, lds_hist, s>>>(
                src, table, sel, hist1d);
        else
            hist1_kernel<DTYPE, kHistWindow, kHistNetThreads>
                <<<cus * (kHistThreads / kHistNetThreads), kHistNetThreads,
                   kHistWindow * sizeof(uint32_t), s>>>(src, table, sel, hist1d);
    }
    if (DTYPE == kF32) {
        if (p->total_sc) {
            ProfileScope ps("hist2c", s);
            hist2c_kernel<<<cus * 4, 256, 0, s>>>(table, sel, cand, chunk_info, uint32_t(n_slots),
                                                  p->cand_cap, hist2);
        }
        {
            ProfileScope ps("hist2", s);
            hist2_kernel<<<cus * 8, 256, 0, s>>>(src, table, sel, hist2);
        }
        {
            ProfileScope ps("select2", s);
            select2_kernel<<<L, kHistThreads, 0, s>>>(table, hist2, sel);
        }
    }
    {
        // the plan fixed the compaction tile's height, and with it which kernels these are
        // (and whether chunks hold dozens or hundreds of candidates)
        const bool rows4 = p->compact_rows == 4, wd = p->emit_wide;
        auto count = wd ? (rows4 ? count_kernel<DTYPE, 4, true> : count_kernel<DTYPE, 2, true>)
                        : (rows4 ? count_kernel<DTYPE, 4, false> : count_kernel<DTYPE, 2, false>);
        auto place = wd ? (rows4 ? place_kernel<DTYPE, 4, true> : place_kernel<DTYPE, 2, true>)
                        : (rows4 ? place_kernel<DTYPE, 4, false> : place_kernel<DTYPE, 2, false>);
        const int occ = resident_blocks_per_cu(place, kEmitThreads, 0, &occ_place[wd][rows4]);
        if (occ <= 0) return TAGC_EHIP;
        // emit_body: kEmitItems super-chunks per workgroup; emit_wide_body: one per wave
        const uint32_t per_wg = wd ? kEmitThreads / 64 : uint32_t(kEmitItems);
        const uint32_t n_emit = (p->total_sc + per_wg - 1) / per_wg;
        // Dense route: one tile per workgroup when dense-route work is certain.  When no
        // segment is planned for this route the part is only a safety net for re-routed
        // segments and nearly always exits at once: a grid that fits the device takes the
        // tiles in turns then.
        const uint32_t n_compact =
            p->static_dense ? p->total_tiles
                            : std::min<uint32_t>(p->total_tiles, uint32_t(cus) * uint32_t(occ));
        {
            ProfileScope ps("count", s);
            count<<<n_emit + n_compact, kEmitThreads, 0, s>>>(
                n_emit, src, table, sel, cand, chunk_info, n_slots, p->cand_cap, sc_cnt, tile_cnt,
                group_cnt);
        }
        {
            ProfileScope ps("place", s);
            place<<<n_emit + n_compact, kEmitThreads, 0, s>>>(
                n_emit, src, table, sel, cand, chunk_info, n_slots, p->cand_cap, sc_cnt, tile_cnt,
                group_cnt, rk->idx, rk->val, bitmap1, rk->cnt);
        }
    }
    if (wide && p->n_c) {
        ProfileScope ps("widen4", s);
        const uint32_t n_words = uint32_t(p->n_c / 32);
        widen4_kernel<<<(n_words + 255) / 256, 256, 0, s>>>(bitmap1, n_words, rk->bitmap);
    }
    return hip_ok(hipGetLastError());
}

}  // namespace

int launch_feedback_apply(const tagc_plan_t *p, const tagc_rank_buffers *rk,
                          const tagc_shared_buffers *sh, hipStream_t s)
{
    const uint32_t n_words = uint32_t(p->n_c / 32);
    if (!n_words) return TAGC_OK;
    ProfileScope ps("feedback_apply", s);
    const SentMap sent{rk->bitmap, p->cfg.index_mode == TAGC_INDEX_ADD4 ? 1u : 0u};
    feedback_apply_kernel<<<(n_words + 255) / 256, 256, 0, s>>>(
        static_cast<const uint32_t *>(sh->table), sent, n_words, static_cast<char *>(rk->acc),
        p->cfg.dtype == TAGC_BF16 ? kBF16 : kF32);
    return hip_ok(hipGetLastError());
}

int launch_sparsify(const tagc_plan_t *p, const void *grad, const tagc_rank_buffers *rk,
                    const tagc_shared_buffers *sh, hipStream_t s)
{
    return p->cfg.dtype == TAGC_BF16 ? launch_sparsify_t<kBF16>(p, grad, rk, sh, s)
                                     : launch_sparsify_t<kF32>(p, grad, rk, sh, s);
}

// ------------------------------------------------ workspace without a caller
//
// For callers that cannot hand over (or allocate) a rank workspace: the same kernels work
// on this array instead.  In host code `scratch` is only a stand-in for the symbol, not a
// device address; the address on the current device is looked up once per device and kept.
// Every GPU holds its own copy of the array at its own address until the process ends.
static __device__ __align__(256) unsigned char scratch[TAGC_STATIC_WORKSPACE_BYTES];

int static_workspace(void **out)
{
    static std::mutex mu;
    static void *ptr[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TAGC_EHIP;
    std::lock_guard<std::mutex> lk(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TAGC_EHIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return TAGC_OK;
}

}  // namespace tagc
