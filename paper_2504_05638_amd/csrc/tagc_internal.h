// Internal declarations shared by the libtagc sources (host plan + HIP kernels).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <vector>

#include "tagc.h"

namespace tagc {

// ---------------------------------------------------------------- constants

constexpr uint32_t kBins1 = 32768;   // top 15 key bits: all of a bf16 key, key>>16 of fp32
constexpr uint32_t kBins2 = 65536;   // low 16 key bits (fp32 only)
constexpr uint32_t kHistThreads = 1024;
constexpr uint32_t kCompactThreads = 256;
constexpr uint32_t kCandRows = 4;        // 16-byte vectors per lane per candidate chunk
constexpr uint32_t kCandChunksPerSuper = 32;  // chunks one emit workgroup handles
constexpr uint32_t kEmitThreads = 256;
constexpr int kEmitItems = 2;  // super-chunks per workgroup of the candidate route's last pass
constexpr uint32_t kSampleVectors = 4096;     // 16-byte vectors sampled per segment
constexpr uint32_t kFastMinElems = 1u << 17;  // shorter segments take the dense path
constexpr uint32_t kFastMinKeep = 64;
constexpr uint32_t kWideEmitCap = 192;  // candidate slots per chunk from which count / place give a wave to a super-chunk
constexpr uint32_t kWideEmitSuperChunks = 2048;  // ... and super-chunks per bucket from which they do so anyway
constexpr double kFastMaxCandFrac = 0.30;  // expected candidates per element beyond which the dense path is planned
constexpr uint32_t kChunkWords = 1024;  // Index words per popcount chunk
constexpr uint32_t kTileGroup = 64;     // dense-route tiles whose counts are also kept as one sum
// A partition keeps, in LDS, 10 bytes per cell (value, meta word, queue slot) and 4 per
// unknown (its c-index): 12288 cells and 8192 unknowns fill the 160 KiB.
constexpr uint32_t kDefaultPartCells = 12288;
constexpr uint32_t kDefaultPartUnknowns = 8192;
constexpr uint32_t kMaxPartCells = 16383;      // 16 queue sweeps of 1024 threads at most
constexpr uint32_t kMaxPartUnknowns = 16384;   // local ranks fit 14 bits
constexpr uint32_t kDecodeThreads = 1024;
constexpr uint32_t kLdsBytes = 160 * 1024;
constexpr uint32_t kMaxRanksPerPass = 32;
// Candidate histogram of the single-read route: the bins from a segment's pre-threshold
// upwards (12 octaves of magnitude: a gradient may grow 4000-fold between two calls before
// its threshold leaves the window); then one count of everything above them, one of the
// non-finite entries, padding.
constexpr uint32_t kWinBins = 1536;
constexpr uint32_t kWinWords = 1544;

// Device copy of one compressed segment.
struct SegDev {
    uint64_t offset;      // element offset in the gradient buffer
    uint32_t n;           // elements
    uint32_t c_off;       // c-index of element 0 (multiple of 32)
    uint32_t k;           // keep count
    uint32_t tile_start;  // first compaction tile of this segment (dense path)
    uint32_t flags;       // kSegAligned | kSegFast
    uint32_t sc_start;    // first super-chunk of this segment (candidate path)
};
constexpr uint32_t kSegAligned = 1;  // offset is a multiple of the 16-byte vector
constexpr uint32_t kSegFast = 2;     // eligible for the single-read candidate path
static_assert(sizeof(SegDev) == 32, "SegDev layout");

// Result of the threshold search for one segment (device memory).  Written for every
// segment with k > 0 and n > 0: by the scan's last workgroup on the segment, by the dense
// route's selection, and (fp32) completed by the second-level selection.
struct SelDev {
    uint32_t T;       // threshold key; keep key > T, and `quota` lowest-position ties
    uint32_t quota;   // ties (key == T) to keep
    uint32_t G;       // count(key > T)
    uint32_t cnt;     // pairs this segment emits = G + min(E, quota)
    uint32_t bin1;    // fp32: level-1 bin that holds T
    uint32_t G1;      // fp32: count of keys in higher level-1 bins
    uint32_t need2;   // fp32: 1 if the low 16 bits still have to be searched
    uint32_t route;   // 0: candidate path, 1: dense path (by plan, or after a miss)
};
static_assert(sizeof(SelDev) == 32, "SelDev layout");

struct RankPtrs {
    const void *p[kMaxRanksPerPass];
};

// ------------------------------------------------------------------- plan

struct Workspace {  // byte offsets inside a rank workspace
    uint64_t hist1d, hist2, group_cnt;  // cleared by every PHASE_INDEX call before they are added to
    uint64_t sel, tile_cnt, sc_cnt, chunk_info, cand, bitmap1, total;
};

// Device state of a plan, kept behind the segment rows of its table: all zero after
// tagc_plan_upload, and every PHASE_INDEX call leaves it as it found it except for the
// pre-thresholds, which are what is carried from call to call.  It lives with the table and
// not in a rank workspace because nobody but the library writes the table: counters that
// have to start at zero can rely on it without a clearing pass per call.
struct TableState {
    uint32_t *hint;      // [L] pre-threshold bin for the next call, 0 = none
    uint32_t *watch;     // [L] calls that still follow the falling trend after a miss
    uint32_t *prev;      // [L] the bin above which 1.3 k entries lay at the last call
    uint32_t *arrive;    // [L] workgroups of the scan that are done with the segment
    uint32_t *arrive_d;  // [L] the same for the dense route's histogram
    uint32_t *raised;    // [L] highest pre-threshold a wave of the scan used
    uint32_t *reroute;   // [L] a chunk overflowed its slots
    uint32_t *glob;      // [8] flags, non-finite inputs, dense-route segments of the call
    uint32_t *win;       // [L][kWinWords] candidate histograms
};
__host__ __device__ inline TableState table_state(uint32_t *table, uint32_t L)
{
    // behind the 32-byte rows: the histograms (a multiple of 32 bytes each), then the rest
    uint32_t *w = table + 8 + 8 * size_t(L);
    uint32_t *p = w + size_t(L) * kWinWords + 8;
    return TableState{p,         p + L,     p + 2 * L, p + 3 * L, p + 4 * L,
                      p + 5 * L, p + 6 * L, p - 8,     w};
}
static_assert(kWinWords % 8 == 0, "histograms stay 32-byte aligned");
constexpr uint64_t table_state_words(uint64_t L) { return 7 * L + 8 + L * kWinWords; }

}  // namespace tagc

struct tagc_plan_s {
    tagc_config cfg;
    std::vector<tagc_segment> segments;       // as given
    std::vector<tagc::SegDev> table;          // compressed segments only
    uint32_t elem_bytes, vec_elems;
    uint32_t compact_rows;                    // 16-byte vectors per thread per compaction tile (2 or 4)
    uint32_t tile_elems;                      // elements per compaction tile
    uint32_t total_tiles;
    uint32_t total_sc;                        // super-chunks of the candidate path
    uint32_t chunk_elems, cand_cap;           // elements / candidate slots per chunk
    uint32_t cnt_ranges;                      // word offset of the partition ranges in a rank's cnt buffer
    bool any_nonfast;                         // some non-empty segment is never streamed by scan_spill
    bool static_dense;                        // some segment with k > 0 never takes the candidate route
    bool emit_wide;                           // chunks hold hundreds of candidates: a wave per super-chunk in count / place
    uint64_t n_real, n_c, K, U_cap, A_cap, m_cap;
    uint32_t P_cap, T_cap;
    tagc::Workspace ws;
    uint64_t zero_bytes;                      // prefix of the rank workspace cleared per call
    // the table was uploaded and no PHASE_INDEX call has sampled pre-thresholds for it yet
    mutable std::atomic<uint32_t> sample_pending{0};
    uint64_t n_chunks;                        // popcount chunks of the Index
    tagc_sizes sizes;
};

namespace tagc {

// ------------------------------------------------------------------- hash

__host__ __device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

__host__ __device__ inline uint32_t seed_word(uint64_t seed, uint32_t j)
{
    return mix32(uint32_t(seed) ^ mix32(uint32_t(seed >> 32) + 0x9E3779B9u * (j + 1)));
}

// slot in [0, m_sub) in the upper bits, sign flag (1 = negative) in bit 31... returned
// separately: slot via multiply-shift range reduction, sign from the low hash bit.
__host__ __device__ inline uint32_t hash_slot(uint32_t i, uint32_t sw, uint32_t m_sub,
                                              uint32_t *neg)
{
    uint32_t h = mix32(i ^ sw);
    *neg = h & 1u;
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(h, m_sub);
#else
    return uint32_t((uint64_t(h) * m_sub) >> 32);
#endif
}

// ---------------------------------------------------------------- profile

void profile_begin(const char *name, hipStream_t s);
void profile_end(hipStream_t s);

struct ProfileScope {
    hipStream_t s;
    ProfileScope(const char *name, hipStream_t st) : s(st) { profile_begin(name, st); }
    ~ProfileScope() { profile_end(s); }
};

int device_cu_count();

// ------------------------------------------------------ stage entry points

int launch_sparsify(const tagc_plan_t *p, const void *grad, const tagc_rank_buffers *rk,
                    const tagc_shared_buffers *sh, hipStream_t s);
int launch_feedback_apply(const tagc_plan_t *p, const tagc_rank_buffers *rk,
                          const tagc_shared_buffers *sh, hipStream_t s);
int launch_encode(const tagc_plan_t *p, const tagc_rank_buffers *rk,
                  const tagc_shared_buffers *sh, hipStream_t s);
int launch_index_or(const tagc_plan_t *p, const tagc_rank_buffers *ranks, uint32_t n_ranks,
                    const tagc_shared_buffers *sh, hipStream_t s);
int launch_sketch_sum(const tagc_plan_t *p, const tagc_rank_buffers *ranks, uint32_t n_ranks,
                      const tagc_shared_buffers *sh, hipStream_t s);
int launch_decode(const tagc_plan_t *p, const tagc_shared_buffers *sh,
                  const tagc_rank_buffers *ranks, uint32_t n_ranks, uint32_t *idx_out,
                  float *val_out, float *dense_out, hipStream_t s);

size_t decode_lds_bytes(uint32_t T_cap, uint32_t P_cap);
size_t salt_lds_bytes(uint32_t T_cap, uint32_t P_cap);

// device address, on the current device, of the library's own rank workspace
// (TAGC_STATIC_WORKSPACE_BYTES); looked up on the first call per device, never allocated
int static_workspace(void **out);

inline int hip_ok(hipError_t e) { return e == hipSuccess ? TAGC_OK : TAGC_EHIP; }

}  // namespace tagc
