// Host side of libtagc: plan construction, size accounting, argument checks and the
// extern "C" entry points.  No kernel lives here.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "tagc_internal.h"
#include "tagc_test.h"

using namespace tagc;

namespace {

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
uint64_t round_up(uint64_t a, uint64_t b) { return ceil_div(a, b) * b; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int tagc_plan(const tagc_config *cfg, const tagc_segment *segs, uint32_t n_seg,
                         tagc_plan_t **out)
{
    if (!cfg || !out || (n_seg && !segs)) return TAGC_EINVAL;
    *out = nullptr;
    if (cfg->dtype != TAGC_F32 && cfg->dtype != TAGC_BF16) return TAGC_EINVAL;
    if (cfg->n_hash != 3 || cfg->n_ranks == 0 || cfg->sizing_milli == 0) return TAGC_EINVAL;
    if (cfg->sizing != TAGC_SIZE_LOAD_FACTOR && cfg->sizing != TAGC_SIZE_FIXED_RATIO)
        return TAGC_EINVAL;
    if (cfg->index_mode > TAGC_INDEX_ADD4) return TAGC_EUNSUPPORTED;
    if (cfg->decode_mode > TAGC_DECODE_ESTIMATE || cfg->cell_type > TAGC_CELL_BF16 ||
        cfg->reserved != 0)
        return TAGC_EINVAL;
    uint32_t P_cap = cfg->part_unknowns ? cfg->part_unknowns : kDefaultPartUnknowns;
    uint32_t T_cap = cfg->part_cells ? cfg->part_cells : kDefaultPartCells;
    if (P_cap > kMaxPartUnknowns || T_cap > kMaxPartCells || T_cap < 3 || T_cap % 3 ||
        decode_lds_bytes(T_cap, P_cap) + 64 > kLdsBytes)
        return TAGC_EINVAL;

    tagc_plan_t *p = new (std::nothrow) tagc_plan_s();
    if (!p) return TAGC_ENOMEM;
    p->cfg = *cfg;
    p->P_cap = P_cap;
    p->T_cap = T_cap;
    p->elem_bytes = cfg->dtype == TAGC_F32 ? 4 : 2;
    p->vec_elems = 16 / p->elem_bytes;
    p->chunk_elems = 64 * p->vec_elems * kCandRows;
    p->cand_cap = 32;
    p->static_dense = false;
    p->any_nonfast = false;

    // Candidate route: slots per chunk for 1.3 x the kept fraction plus six standard
    // deviations.  What follows the scan costs in proportion to the candidates; with the
    // form of count and place that suits the number of candidates per chunk (emit_body for
    // dozens, emit_wide_body for hundreds) it beats the dense route's three reads of the
    // gradient up to Table 1's 2x regime (a fifth kept: 26 % of a chunk expected as
    // candidates; measured on 7B-shaped buckets).  Returns the slots a chunk needs, 0 = dense
    // route.
    auto fast_slots = [&](const tagc_segment &s) -> uint32_t {
        const uint64_t k = uint64_t((unsigned __int128)s.length * s.keep_ppm / 1000000u);
        if (s.offset % p->vec_elems || s.length < kFastMinElems || k < kFastMinKeep) return 0;
        const double mu = 1.3 * double(k) / double(s.length) * p->chunk_elems;
        if (mu > kFastMaxCandFrac * p->chunk_elems) return 0;
        return uint32_t(round_up(uint64_t(mu + 6.0 * sqrt(mu) + 16.0), 32));
    };
    // Compaction tile of the dense route: four 16-byte vectors per thread where that route
    // is planned work, two where it is only the safety net of re-routed segments -- the
    // kernel it shares with the candidate route's last pass then needs few enough
    // registers for one more workgroup per CU.
    for (uint32_t l = 0; l < n_seg; ++l) {
        const tagc_segment &s = segs[l];
        if (!(s.flags & TAGC_SEG_COMPRESS) || s.keep_ppm > 1000000u || s.length == 0) continue;
        if ((unsigned __int128)s.length * s.keep_ppm / 1000000u && !fast_slots(s))
            p->static_dense = true;
    }
    p->compact_rows = p->static_dense ? 4 : 2;
    p->tile_elems = kCompactThreads * p->vec_elems * p->compact_rows;

    uint64_t c = 0, n_real = 0, K = 0, tiles = 0, grad_elems = 0, scs = 0;
    try {
        p->segments.assign(segs, segs + n_seg);
        for (uint32_t l = 0; l < n_seg; ++l) {
            const tagc_segment &s = segs[l];
            if (!(s.flags & TAGC_SEG_COMPRESS)) continue;
            if (s.keep_ppm > 1000000u) {
                delete p;
                return TAGC_EINVAL;
            }
            if (s.length >= (1ull << 31) || c + s.length >= (1ull << 32) ||
                tiles >= (1ull << 31)) {
                delete p;
                return TAGC_ESIZE;
            }
            SegDev d{};
            d.offset = s.offset;
            d.n = uint32_t(s.length);
            d.c_off = uint32_t(c);
            d.k = uint32_t((unsigned __int128)s.length * s.keep_ppm / 1000000u);
            d.tile_start = uint32_t(tiles);
            d.flags = (s.offset % p->vec_elems) == 0 ? kSegAligned : 0;
            if (const uint32_t cap = fast_slots(s)) {
                d.flags |= kSegFast;
                p->cand_cap = std::max(p->cand_cap, cap);
            }
            if (d.n && !(d.flags & kSegFast)) p->any_nonfast = true;
            d.sc_start = uint32_t(scs);
            scs += ceil_div(s.length, uint64_t(p->chunk_elems) * kCandChunksPerSuper);
            p->table.push_back(d);
            c = round_up(c + s.length, 32);
            n_real += s.length;
            grad_elems = std::max(grad_elems, s.offset + s.length);
            K += d.k;
            tiles += ceil_div(s.length, p->tile_elems);
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return TAGC_ENOMEM;
    }
    if (c >= (1ull << 32)) {
        delete p;
        return TAGC_ESIZE;
    }
    // count / place give a wave to every super-chunk where chunks hold hundreds of
    // candidates, and in large buckets whatever they hold: that form needs next to no LDS, so
    // its workgroups run beside another bucket's scan, which is what large buckets are timed
    // with (7B-shaped buckets, 12 in flight: 4 % of a step; one bucket at a time it is 3 us
    // per rank slower than four threads per chunk, which small buckets, bound by the time
    // a launch takes, would notice)
    p->emit_wide = p->cand_cap >= kWideEmitCap || scs >= kWideEmitSuperChunks;
    p->n_real = n_real;
    p->n_c = c;
    p->K = K;
    p->total_tiles = uint32_t(tiles);
    p->total_sc = uint32_t(scs);
    p->U_cap = std::min<uint64_t>(n_real, uint64_t(cfg->n_ranks) * K);
    uint64_t M_max = cfg->sizing == TAGC_SIZE_LOAD_FACTOR
                         ? ceil_div(uint64_t(cfg->sizing_milli) * p->U_cap, 1000)
                         : ceil_div(n_real * 1000, cfg->sizing_milli);
    uint64_t q = T_cap / 3;
    p->A_cap = std::max<uint64_t>(1, std::max(ceil_div(p->U_cap, P_cap), ceil_div(M_max, 3 * q)));
    p->m_cap = M_max + 3 * p->A_cap + 3;
    if (p->m_cap >= (1ull << 32) || p->A_cap >= (1ull << 31)) {
        delete p;
        return TAGC_ESIZE;
    }
    const uint64_t L = p->table.size();
    const uint64_t words = p->n_c / 32;
    p->n_chunks = ceil_div(words, kChunkWords);

    // rank workspace: the histograms that are added to by atomics (a prefix that every
    // PHASE_INDEX call clears before use), then plain scratch that is written before it is read
    Workspace &w = p->ws;
    const uint64_t chunks = scs * kCandChunksPerSuper;
    if (chunks * p->cand_cap >= (1ull << 32)) {  // slot numbers are kept in 32 bits
        delete p;
        return TAGC_ESIZE;
    }
    uint64_t off = 0;
    w.hist1d = off;
    off += L * kBins1 * 4;
    w.hist2 = off;
    off += (cfg->dtype == TAGC_F32 ? L * kBins2 * 4 : 0);
    w.group_cnt = off;
    off += round_up((tiles / kTileGroup + 1) * 8, 16);
    p->zero_bytes = off;
    w.sel = off;
    off += round_up(L * sizeof(SelDev), 16);
    w.tile_cnt = off;
    off += round_up(tiles * 8, 16);
    w.sc_cnt = off;
    off += round_up(scs * 8, 16);
    w.chunk_info = off;  // per chunk: candidates found, first slot
    off += round_up(chunks * 8, 16);
    off = round_up(off, 128);  // a chunk's slots then start on a cache-line boundary
    w.cand = off;
    off += round_up(chunks * p->cand_cap * (cfg->dtype == TAGC_F32 ? 8 : 4), 16);
    w.bitmap1 = off;  // 4-bit Index: the 1-bit Index is built here and widened from here
    if (cfg->index_mode == TAGC_INDEX_ADD4) off += round_up(4 * words, 16);
    w.total = std::max<uint64_t>(off, 16);

    tagc_sizes &z = p->sizes;
    memset(&z, 0, sizeof(z));
    z.n_seg_compressed = L;
    z.n_real = n_real;
    z.n_c = p->n_c;
    z.bitmap_words = words;
    z.pair_capacity = K;
    z.union_capacity = p->U_cap;
    z.partition_capacity = p->A_cap;
    z.sketch_cells_capacity = p->m_cap;
    z.part_unknowns = P_cap;
    z.part_cells = T_cap;
    z.grad_elems = grad_elems;
    // header, one row per compressed segment, then the plan's device state (pre-thresholds,
    // arrival counters, candidate histograms: see TableState)
    z.table_bytes = 32 + 32 * std::max<uint64_t>(L, 1) +
                    round_up(4 * table_state_words(std::max<uint64_t>(L, 1)), 16);
    z.rank_idx_bytes = round_up(4 * std::max<uint64_t>(K, 1), 16);
    z.rank_val_bytes = z.rank_idx_bytes;
    // counts first, then (from the Index aggregation on) the A+1 positions at which the
    // rank's sorted pair list crosses the partition bounds
    p->cnt_ranges = uint32_t(round_up(TAGC_CNT_SEG0 + L, 4));
    z.rank_cnt_bytes = round_up(4 * (p->cnt_ranges + p->A_cap + 2), 16);
    const uint64_t wire = cfg->index_mode == TAGC_INDEX_ADD4 ? 4 : 1;  // bits per parameter
    z.rank_bitmap_bytes = round_up(4 * wire * std::max<uint64_t>(words, 1), 16);
    const uint64_t cell_bytes = cfg->cell_type == TAGC_CELL_BF16 ? 2 : 4;  // on the wire
    // (one partition of slack behind the cells: tagc_reduce_decompress reads whole tiles
    // of the default partition size from a partition's first cell on, and stages only the
    // partition's own cells)
    z.rank_sketch_bytes = round_up(cell_bytes * p->m_cap, 16) +
                          (p->cfg.cell_type == TAGC_CELL_F32 ? 4ull * kDefaultPartCells : 0ull);
    z.rank_workspace_bytes = w.total;
    z.shared_bitmap_bytes = round_up(4 * std::max<uint64_t>(words, 1), 16);
    z.shared_sketch_bytes = round_up(4 * p->m_cap, 16);
    z.shared_header_bytes = 4 * TAGC_HDR_WORDS;
    // the partitions' first c-indices (A + 1), then their hash salts (A)
    z.shared_bounds_bytes = round_up(4 * (2 * p->A_cap + 1), 16);
    // chunk prefixes; behind them, when the 4-bit Index of more ranks than one pass takes is
    // summed, the running 4-bit sum
    z.shared_workspace_bytes = round_up(4 * (p->n_chunks + 1), 16);
    if (cfg->index_mode == TAGC_INDEX_ADD4 && cfg->n_ranks > kMaxRanksPerPass)
        z.shared_workspace_bytes += round_up(16 * words, 16);
    z.shared_status_bytes = 4 * TAGC_ST_WORDS;
    z.out_idx_bytes = round_up(4 * std::max<uint64_t>(p->U_cap, 1), 16);
    z.out_val_bytes = z.out_idx_bytes;
    z.out_dense_bytes = round_up(4 * std::max<uint64_t>(p->n_c, 1), 16);
    if (n_real) {
        z.wire_index_bits = 2.0 * double(wire) * double(p->n_c) / double(n_real);
        double cells = cfg->sizing == TAGC_SIZE_LOAD_FACTOR ? double(p->m_cap) : double(M_max);
        z.wire_sketch_bits = 8.0 * double(cell_bytes) * cells / double(n_real);
        z.wire_total_bits = z.wire_index_bits + z.wire_sketch_bits;
    }
    *out = p;
    return TAGC_OK;
}

extern "C" void tagc_plan_destroy(tagc_plan_t *p) { delete p; }

extern "C" int tagc_plan_sizes(const tagc_plan_t *p, tagc_sizes *out)
{
    if (!p || !out) return TAGC_EINVAL;
    *out = p->sizes;
    return TAGC_OK;
}

extern "C" int tagc_plan_upload(const tagc_plan_t *p, void *table_dev, void *stream)
{
    if (!p || !table_dev || !aligned16(table_dev)) return TAGC_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t hdr[8] = {uint32_t(p->table.size()), p->total_tiles, uint32_t(p->n_c),
                       uint32_t(p->n_chunks), p->total_sc, 0, 0, 0};
    // Two small copies from pageable host memory: hipMemcpyAsync stages them before it
    // returns, so `hdr` may live on this stack frame.
    if (hipMemcpyAsync(table_dev, hdr, sizeof(hdr), hipMemcpyHostToDevice, s) != hipSuccess)
        return TAGC_EHIP;
    if (!p->table.empty() &&
        hipMemcpyAsync(static_cast<char *>(table_dev) + 32, p->table.data(),
                       p->table.size() * sizeof(SegDev), hipMemcpyHostToDevice,
                       s) != hipSuccess)
        return TAGC_EHIP;
    // the plan's device state starts at zero; no pre-threshold is known yet, so the first
    // PHASE_INDEX call samples
    if (!p->table.empty() &&
        hipMemsetAsync(static_cast<char *>(table_dev) + 32 + p->table.size() * sizeof(SegDev), 0,
                       4 * table_state_words(p->table.size()), s) != hipSuccess)
        return TAGC_EHIP;
    p->sample_pending.store(1, std::memory_order_relaxed);
    return TAGC_OK;
}

static int check_rank(const tagc_rank_buffers *r)
{
    if (!r || !r->idx || !r->val || !r->cnt || !r->bitmap || !r->sketch || !r->workspace)
        return TAGC_EINVAL;
    if (!aligned16(r->idx) || !aligned16(r->val) || !aligned16(r->cnt) ||
        !aligned16(r->bitmap) || !aligned16(r->sketch) || !aligned16(r->workspace))
        return TAGC_EINVAL;
    if (r->acc && !aligned16(r->acc)) return TAGC_EINVAL;
    return TAGC_OK;
}

static int check_shared(const tagc_shared_buffers *s)
{
    if (!s || !s->table || !s->bitmap || !s->sketch || !s->header || !s->bounds ||
        !s->workspace || !s->status)
        return TAGC_EINVAL;
    if (!aligned16(s->table) || !aligned16(s->bitmap) || !aligned16(s->sketch) ||
        !aligned16(s->header) || !aligned16(s->bounds) || !aligned16(s->workspace) ||
        !aligned16(s->status))
        return TAGC_EINVAL;
    return TAGC_OK;
}

extern "C" int tagc_compress(const tagc_plan_t *p, uint32_t phase, const void *grad,
                             const tagc_rank_buffers *rk, const tagc_shared_buffers *sh,
                             void *stream)
{
    if (!p) return TAGC_EINVAL;
    int rc = check_rank(rk);
    if (rc) return rc;
    rc = check_shared(sh);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (phase == TAGC_PHASE_INDEX) {
        if (!grad || !aligned16(grad)) return TAGC_EINVAL;
        return launch_sparsify(p, grad, rk, sh, s);
    }
    if (phase == TAGC_PHASE_SKETCH) return launch_encode(p, rk, sh, s);
    return TAGC_EINVAL;
}

extern "C" int tagc_compress_static(const tagc_plan_t *p, uint32_t phase, const void *grad,
                                    const tagc_rank_buffers *rk, const tagc_shared_buffers *sh,
                                    void *stream)
{
    if (!p || !rk) return TAGC_EINVAL;
    if (p->sizes.rank_workspace_bytes > TAGC_STATIC_WORKSPACE_BYTES) return TAGC_ESIZE;
    tagc_rank_buffers r = *rk;
    r.workspace = nullptr;
    const int rc = static_workspace(&r.workspace);
    if (rc) return rc;
    return tagc_compress(p, phase, grad, &r, sh, stream);
}

extern "C" int tagc_feedback_apply(const tagc_plan_t *p, const tagc_rank_buffers *rk,
                                   const tagc_shared_buffers *sh, void *stream)
{
    if (!p || !rk || !rk->acc) return TAGC_EINVAL;
    int rc = check_shared(sh);
    if (rc) return rc;
    rc = check_rank(rk);
    if (rc) return rc;
    return launch_feedback_apply(p, rk, sh, static_cast<hipStream_t>(stream));
}

extern "C" int tagc_aggregate(const tagc_plan_t *p, uint32_t phase,
                              const tagc_rank_buffers *ranks, uint32_t n_ranks,
                              const tagc_shared_buffers *sh, void *stream)
{
    if (!p || !ranks || n_ranks == 0 || n_ranks > p->cfg.n_ranks) return TAGC_EINVAL;
    int rc = check_shared(sh);
    if (rc) return rc;
    for (uint32_t r = 0; r < n_ranks; ++r) {
        rc = check_rank(&ranks[r]);
        if (rc) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (phase == TAGC_PHASE_INDEX) return launch_index_or(p, ranks, n_ranks, sh, s);
    if (phase == TAGC_PHASE_SKETCH) return launch_sketch_sum(p, ranks, n_ranks, sh, s);
    return TAGC_EINVAL;
}

extern "C" int tagc_decompress(const tagc_plan_t *p, const tagc_shared_buffers *sh,
                               uint32_t *idx_out, float *val_out, float *dense_out,
                               void *stream)
{
    if (!p || !idx_out || !val_out) return TAGC_EINVAL;
    int rc = check_shared(sh);
    if (rc) return rc;
    if (!aligned16(idx_out) || !aligned16(val_out) || (dense_out && !aligned16(dense_out)))
        return TAGC_EINVAL;
    return launch_decode(p, sh, nullptr, 0, idx_out, val_out, dense_out,
                         static_cast<hipStream_t>(stream));
}

extern "C" int tagc_reduce_decompress(const tagc_plan_t *p, const tagc_rank_buffers *ranks,
                                      uint32_t n_ranks, const tagc_shared_buffers *sh,
                                      uint32_t *idx_out, float *val_out, float *dense_out,
                                      void *stream)
{
    if (!p || !ranks || n_ranks == 0 || n_ranks > p->cfg.n_ranks || !idx_out || !val_out)
        return TAGC_EINVAL;
    // float32 cells, the default partition size at most, and as many ranks as fit the
    // kernel's argument list
    if (n_ranks > kMaxRanksPerPass || p->cfg.cell_type != TAGC_CELL_F32 ||
        p->T_cap > kDefaultPartCells || p->P_cap > kDefaultPartUnknowns)
        return TAGC_EUNSUPPORTED;
    int rc = check_shared(sh);
    if (rc) return rc;
    for (uint32_t r = 0; r < n_ranks; ++r) {
        rc = check_rank(&ranks[r]);
        if (rc) return rc;
    }
    if (!aligned16(idx_out) || !aligned16(val_out) || (dense_out && !aligned16(dense_out)))
        return TAGC_EINVAL;
    return launch_decode(p, sh, ranks, n_ranks, idx_out, val_out, dense_out,
                         static_cast<hipStream_t>(stream));
}

extern "C" void tagc_hash_host(uint32_t i, uint64_t seed, uint32_t j, uint32_t salt,
                               uint32_t m_sub, uint32_t *slot, int32_t *sign)
{
    uint32_t neg;
    *slot = hash_slot(i, seed_word(seed, j + 3 * salt), m_sub, &neg);
    *sign = neg ? -1 : 1;
}

extern "C" const char *tagc_strerror(int err)
{
    switch (err) {
        case TAGC_OK: return "ok";
        case TAGC_EINVAL: return "invalid argument";
        case TAGC_ESIZE: return "size exceeds what the format can address";
        case TAGC_EUNSUPPORTED: return "not supported";
        case TAGC_EHIP: return "HIP runtime error";
        case TAGC_ENOMEM: return "out of host memory";
        default: return "unknown error";
    }
}
