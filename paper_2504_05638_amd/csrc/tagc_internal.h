// Internal declarations shared by the libtagc sources (host plan + HIP kernels).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
constexpr double kFastMaxCandFrac = 0.04;  // expected candidates per element beyond which the dense path wins
constexpr uint32_t kChunkWords = 1024;  // Index words per popcount chunk
// A partition keeps, in LDS, 10 bytes per cell (value, meta word, queue slot) and 4 per
// unknown (its c-index): 12288 cells and 8192 unknowns fill the 160 KiB.
constexpr uint32_t kDefaultPartCells = 12288;
constexpr uint32_t kDefaultPartUnknowns = 8192;
constexpr uint32_t kMaxPartCells = 16383;      // 16 queue sweeps of 1024 threads at most
constexpr uint32_t kMaxPartUnknowns = 16384;   // local ranks fit 14 bits
constexpr uint32_t kDecodeThreads = 1024;
constexpr uint32_t kLdsBytes = 160 * 1024;
constexpr uint32_t kMaxRanksPerPass = 32;
// polls (about half a microsecond each) for a count another workgroup is expected to
// publish before the waiting one computes it itself.  Far longer than a running workgroup
// takes to count even with the device shared (with 512 polls a run with error feedback
// recomputed tens of thousands of counts that were merely late, each at many times the cost
// of waiting; with 4096 none), short against what a workgroup that has not started can take
constexpr uint32_t kHelpAfterPolls = 1u << 12;
uint32_t help_after_polls();  // kHelpAfterPolls unless a test lowered it

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

// Result of the threshold search for one segment (device memory).
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
    uint64_t hist1, hist1d, hist2, tile_state, sc_state, counters;  // cleared per call
    uint64_t sel, binlo, chunk_cnt, cand, bitmap1, total;
};


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
    uint64_t n_real, n_c, K, U_cap, A_cap, m_cap;
    uint32_t P_cap, T_cap;
    tagc::Workspace ws;
    uint64_t zero_bytes;                      // prefix of the rank workspace cleared per call
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
int launch_decode(const tagc_plan_t *p, const tagc_shared_buffers *sh, uint32_t *idx_out,
                  float *val_out, float *dense_out, hipStream_t s);

size_t decode_lds_bytes(uint32_t T_cap, uint32_t P_cap);
size_t salt_lds_bytes(uint32_t T_cap, uint32_t P_cap);

// device address, on the current device, of the library's own rank workspace
// (TAGC_STATIC_WORKSPACE_BYTES); looked up on the first call per device, never allocated
int static_workspace(void **out);

inline int hip_ok(hipError_t e) { return e == hipSuccess ? TAGC_OK : TAGC_EHIP; }

}  // namespace tagc
