// gravac.hip - Top-k + error-feedback gradient compression for MI355X (gfx950).
//
// Implements the C ABI of include/gravac.h.  The path follows GraVAC (arxiv 2305.12201):
// error feedback (Sec. III-B), Top-k sparsification at a compression factor (Sec. II-C),
// residual update (Alg. 1), compression gain for several candidate CFs (Sec. III-B
// equation, Alg. 1 gain steps), layerwise mode and decompression (Sec. III-A).
//
// Design in one paragraph.  Keys are the binary32 bit patterns of |acc|, so magnitude order is
// unsigned-integer order.  A small stratified sample of acc gives, per candidate CF, a bracket
// [lo, top) of keys that holds the k-th largest key with a statistical safety margin.  ONE streaming
// pass then reads grad and residual, writes acc back as the provisional residual, sums acc^2, and for
// every CF counts (and sums the energy of) the entries above the bracket and histograms the entries
// inside it.  The few entries inside some bracket go, in index order, into a per-sub-tile bracket list;
// the entries that can belong to the committed selection go into a per-sub-tile candidate list, unless
// the sub-tile is mostly candidates, in which case the emit step reads it again from the residual.
// Everything after the pass works on those lists: locate the histogram bin that holds the k-th
// largest, gather the few keys of that bin, resolve the exact key, scan the per-tile counts and emit
// the message in ascending index order while zeroing the selected residual slots.  If a sampled
// bracket turns out wrong the segment is redone by a route that cannot fail: a bin too coarse and too
// full to resolve is binned again inside itself from the bracket lists; a k-th largest outside the
// bracket is found from a 2048-bin histogram of the top key bits of all elements, after which the
// lists are collected again.  Results are identical on every route; only the number of passes over
// memory differs.
//
// Units of work.  A tile is TW consecutive elements; the streaming pass gives each of its SUB
// sub-tiles to one 64-lane wavefront, which owns that sub-tile's slots of the list arrays, so
// ordered compaction needs no communication between wavefronts and no list can overflow.  No kernel
// waits on another workgroup: cross-tile results (histograms, output offsets) are combined at kernel
// boundaries.  Global atomics complete at a rate of roughly one per cache line per 10 ns on this part,
// so the bracket histogram and the gather lists exist in REP copies (picked from the sub-tile,
// tile or workgroup number) and nothing else uses global atomics.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <vector>

#include "gravac.h"
#include "gravac_profile.h"

namespace {

#ifndef GV_TW
#define GV_TW 8192
#endif
constexpr int TW = GV_TW;           // elements per tile (unit of the list kernels)
#ifndef GV_SUB
#define GV_SUB 8
#endif
constexpr int SUB = GV_SUB;         // sub-tiles per tile: the streaming pass gives one wavefront a sub-tile
constexpr int TS = TW / SUB;        // elements per sub-tile
constexpr int WG = 256;             // threads per workgroup of the streaming kernels
constexpr int WAVES = WG / 64;
#ifndef GV_LWG
#define GV_LWG 256
#endif
constexpr int LWG = GV_LWG;         // threads per workgroup of the list kernels (refine, emit)
constexpr int LWAVES = LWG / 64;
constexpr int ROW = 256;            // elements one wavefront touches per load (64 lanes x float4)
constexpr int ROWS = TS / ROW;      // rows of a sub-tile: all of them are in flight together
static_assert(TS % ROW == 0 && ROWS == 4, "a sub-tile is four rows");
#ifndef GV_DENSE
#define GV_DENSE 384
#endif
constexpr uint32_t DENSE_SUB = GV_DENSE;  // a full sub-tile with at least this many candidates keeps no candidate list:
                                          // the emit step reads its 1024 elements again (4 KB read + 4 KB written, what
                                          // about 400 listed candidates cost in list traffic and scattered stores)
constexpr uint32_t DENSE_BIT = 0x80000000u;  // flag of such a sub-tile in cand_cnt
constexpr uint32_t LONG_WALK = 256;   // a tile with at least this many listed entries is walked sub-tile by sub-tile
#ifndef GV_NT
#define GV_NT 1                     // non-temporal hints on the streaming loads and stores
#endif
#ifndef GV_XGRID
#define GV_XGRID 1024
#endif
constexpr uint32_t XGRID = GV_XGRID;  // workgroups of the two exact-route kernels (they loop over the tiles)
constexpr int REP = 8;              // copies of the bracket histogram and of the gather lists
constexpr int NBIN = 2048;          // bins of the bracket / refine / coarse histograms
constexpr uint32_t OVF = NBIN - 1;  // bins 0 .. OVF - 1 cover the bracket; bin OVF stands for everything above it
constexpr uint32_t XBINS = 1024;    // bins in use after an exact route has binned a segment again
constexpr int SBIN = 4096;          // bins of the sample histogram: 2^17 keys each (64 per octave, 1.1 % in magnitude)
constexpr uint32_t SSHIFT = 17;     // from |x| = 2^-48 up to 2^16; smaller magnitudes share bin 0, larger ones the last bin
constexpr uint32_t SKEY0 = 79u << 23;
static_assert((uint64_t)SKEY0 + ((uint64_t)SBIN << SSHIFT) <= 0x7F800000ull, "the window lies inside the finite keys");
constexpr int SGRP = 8;             // the sample bins in SGRP groups: one workgroup of the threshold kernel each
constexpr int SAMPLE_BLOCK = 1024;  // samples per workgroup of the sampling kernel
constexpr int SAMPLE_MAX = 65536;   // samples of a flat tensor at most (unless k n is large, see SAMPLE_MAX_FLAT)
constexpr int SAMPLE_MAX_SEG = 32768;  // layerwise: samples per tensor at most (a tensor of up to twice that is read whole)
constexpr int SAMPLE_MAX_FLAT = 524288;  // flat mode, a large k: see sample_count
constexpr int DENSE_ROUNDS = 4;          // ... whose sample blocks are up to DENSE_ROUNDS * SAMPLE_BLOCK samples each
constexpr int DENSE_BLOCKS = 128;        // ... so that there are at most this many of them
constexpr int LCAP = 4096;          // keys a gather list can hold
constexpr int MAXCF = GRAVAC_MAX_CF;
constexpr double ZMARGIN = 5.0;     // safety margin of the sampled rank, in standard deviations
constexpr uint32_t NONE = 0xFFFFFFFFu;
constexpr uint32_t KEY_END = 0x80000000u;  // one past the largest key

enum : uint32_t { MODE_RESOLVED = 0, MODE_GATHER = 1, MODE_HIST = 2, MODE_FAIL = 3 };
// SegState::fail, the heavier kind over the segment's CFs wins:
//   FAIL_NARROW  the bin that holds the k-th largest is known but too coarse and too full to resolve: only the
//                CFs concerned are binned again, inside that bin, from the bracket lists (no pass over the gradient);
//   FAIL_FULL    the k-th largest lies outside the bracket (or there was none): acc is read again.
enum : uint32_t { FAIL_NONE = 0, FAIL_NARROW = 1, FAIL_FULL = 3 };
// where a call's brackets come from
enum : uint32_t { BOUNDS_SAMPLED = 0, BOUNDS_RANDOM = 1, BOUNDS_FORCED = 2,
                  BOUNDS_FIXED = 3 };  // the threshold sparsifier: the caller gives the threshold, nothing is searched for

// Selection state of one (segment, CF).
struct CfState {
    uint32_t k;         // entries to select
    uint32_t lo;        // first key of the bracket histogram's bin 0
    uint32_t s;         // bin = (key - lo) >> s
    uint32_t mode;      // MODE_*
    uint32_t base;      // first key of the bin that holds the k-th largest
    uint32_t span;      // a key lies in that bin iff 0 <= key - base <= span
    uint32_t above;     // number of keys above that bin
    uint32_t c;         // number of keys in that bin
    uint32_t tau;       // key of the k-th largest (valid once resolved)
    uint32_t need;      // how many keys equal to tau are selected (lowest indices first)
    uint32_t cnt_gt;    // number of keys greater than tau
    uint32_t redo;      // 1 if this CF is binned again on the narrow route (set by the locate step)
    uint32_t lo2, s2;   // ... with these bounds: the located bin, cut into XBINS parts
    uint32_t top;       // the pass over the gradient has counted keys >= top as above the bracket (KEY_END: none)
    uint32_t pad;
};
static_assert(sizeof(CfState) == 64, "CfState layout");

struct SegState {
    uint32_t lo_min;  // smallest lo over the CFs: keys below it concern no CF
    uint32_t fail;    // FAIL_*: whether a bracket failed and the segment takes an exact route, and which
    uint32_t pz;      // sparse sub-tiles: the first pass has stored +0 instead of acc for keys >= pz: the upper end of the
                      // committed CF's bracket, above which an entry is selected unless the bracket fails (NONE: none)
    uint32_t lo_c;    // the committed CF's lo: keys from here on are candidates for the message
};

struct Status {
    int any_fail;
    int n_fail;
    int error;
    int n_seg;
    int n_narrow;             // segments of n_fail that were only binned again from their bracket lists
    int count;                // threshold sparsifier: entries at or above the threshold (written by the scan)
    int pad[2];
};

typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

// One tensor of a layerwise call.
struct SegInfo {
    int64_t begin, end;      // element range in the flat gradient
    int64_t koff;            // offset of the segment's message in out_idx / out_val
    uint32_t tile0, tile1;   // tile range
    uint32_t samp0;          // first sample block
    uint32_t samp_cnt;       // samples taken
    uint32_t small;          // 1: at most SMALL_MAX elements, handled by one workgroup out of LDS: no tiles, no samples
    uint32_t rep;            // copies of the segment's bracket histograms and gather lists: REP for a large tensor, else 1
    uint32_t pool0;          // its first copy block in hist1 / list_* / list_cnt (n_cf * rep consecutive blocks, CF-major)
    uint32_t pad[3];
};
static_assert(sizeof(SegInfo) == 64, "SegInfo layout");

struct Params {
    const float* grad;       // gradient; in single-source mode the values of the level-1 message
    float* res;              // residual (in: leftover, out: acc with the selection zeroed); null in single-source mode
    const float* acc;        // where acc can be re-read after the streaming pass: res, or grad in single-source mode
    const int32_t* map_idx;  // single-source mode: index of every source element in the dense gradient (else null)
    float* restore;          // single-source mode: dense residual that gets the unselected values back (or null)
    int64_t n_restore;       // its length
    int single;              // 1 = single-source mode (second-level compression of a message)
    int random;              // 1 = Random-k: the order is that of a keyed priority of the index, not of |acc|
    int no_commit;           // 1: nothing is removed from the residual (it keeps acc); the caller commits a message later
    int vec_ok;              // 1 if every buffer the kernels read or write with 16-byte accesses is aligned to 16 bytes
    int split;               // 1 if the committed CF is not the lowest of the list: the entries inside the brackets then get a
                             // list of their own everywhere; 0: a sub-tile's candidate list, where it has one, holds them all
    uint32_t bounds_from;    // BOUNDS_*
    uint32_t fixed_key;      // BOUNDS_FIXED: the key of the caller's threshold; entries with key >= fixed_key are kept
    uint32_t rk_s0, rk_s1;   // Random-k: the two 31-bit keys (from the seed)
    int64_t n;
    int n_seg;  // >= 1
    int n_cf;
    int commit;
    int64_t total_out;        // pairs the call emits
    uint32_t n_tiles;
    uint32_t n_sample_blocks;
    // layerwise tables in the workspace (unused when n_seg == 1)
    const SegInfo* segs;           // [n_seg] built on the host
    const uint32_t* ktab;          // [n_seg][n_cf] built on the host
    const uint32_t* sblock_seg;    // [n_sample_blocks] segment of every sample block, built on the host
    const uint32_t* small_list;    // [n_small] the segments handled by one workgroup each, built on the host
    uint32_t n_small;
    uint32_t* tseg;                // [n_tiles] segment of every tile, filled by threshold_kernel
    // the same for one flat tensor
    uint32_t flat_k[MAXCF];
    uint32_t flat_samples;
    // workspace
    Status* status;
    CfState* st;         // [n_seg][n_cf]
    SegState* seg;       // [n_seg]
    uint32_t* bnd_lo;    // [n_seg][n_cf] the bracket of every CF as the threshold kernel found it: first key ...
    uint32_t* bnd_hi;    // [n_seg][n_cf] ... and one past its last key (at most KEY_END)
    uint32_t* bnd_mid;   // [n_seg][n_cf] the key the sample puts the k-th largest at (NONE: no estimate)
    uint32_t* hist1;     // [copy blocks][NBIN] bracket histograms: REP copies per CF of a large tensor, one otherwise
    uint32_t* ovfc;      // [n_seg][n_cf][64][32] counts above the bracket (the histogram's last bin), spread over
                         // 64 cache lines; word 0 of each line is used
    uint32_t* hist2;     // [n_seg][n_cf][NBIN] refine histogram
    uint32_t* coarse;    // [n_seg][NBIN] histogram of key >> 20 (exact route)
    uint32_t* list_key;  // [copy blocks][LCAP] gather lists: key ...
    uint32_t* list_tile; //                          ... tile ...
    float* list_val;     //                          ... and value (written for Random-k only) of the listed entries
    uint32_t* list_cnt;  // [copy blocks][32] fill counts of the gather lists, one cache line each
    uint32_t* samp_hist; // [n_sample_blocks][SBIN / 2] sample histograms, two 16-bit counts per word
    uint32_t* samp_grp;  // [n_sample_blocks][SGRP] samples per group of SBIN / SGRP bins
    uint32_t* cand_cnt;  // [n_tiles][SUB] listed candidates of every sub-tile (| DENSE_BIT: none listed, the sub-tile is read again)
    uint32_t* brk_cnt;   // [n_tiles][SUB] bracket-list entries of every sub-tile
    uint32_t* ovn;       // [n_tiles][SUB][n_cf] entries of the sub-tile above CF j's bracket
    double* ovs;         // [n_tiles][SUB][n_cf] ... and their sum of acc^2
    uint32_t* tg0;       // [n_tiles] entries of the tile above the committed CF's located bin
    uint32_t* tin;       // [n_tiles] entries of the tile inside that bin
    uint32_t* toff;      // [n_tiles] offset of the tile's output inside its segment's message
    uint32_t* ttake;     // [n_tiles] how many of the tile's entries equal to tau(commit) are selected
    uint32_t* tsel;      // [n_tiles] pairs the tile emits
    double* ssd;         // [n_tiles][SUB] sum of acc^2 of every sub-tile
    double* ssd_t;       // [n_tiles] sum of acc^2 of the tile
    double* sss;         // [n_tiles][n_cf] sum of acc^2 over the tile's keys above CF j's located bin
    int32_t* cand_idx;   // [n_tiles][SUB][TS] candidate list: sub-tile j of tile u owns the slots from (u*SUB + j)*TS
    float* cand_val;     // [n_tiles][SUB][TS]
    uint32_t* brk_key;   // [n_tiles][SUB][TS] bracket list: keys ...
    float* brk_val;      // [n_tiles][SUB][TS] ... and values (written for Random-k only)
    // outputs
    int32_t* out_idx;
    float* out_val;
    int64_t* out_count;
    double* out_stats;
};

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ bool is_flat(const Params& p) { return p.n_seg == 1; }
__device__ __forceinline__ int64_t seg_begin(const Params& p, int t) { return is_flat(p) ? 0 : p.segs[t].begin; }
__device__ __forceinline__ int64_t seg_end(const Params& p, int t) { return is_flat(p) ? p.n : p.segs[t].end; }
__device__ __forceinline__ uint32_t seg_tile0(const Params& p, int t) { return is_flat(p) ? 0u : p.segs[t].tile0; }
__device__ __forceinline__ uint32_t seg_tile1(const Params& p, int t) { return is_flat(p) ? p.n_tiles : p.segs[t].tile1; }
__device__ __forceinline__ uint32_t seg_k(const Params& p, int t, int j) { return is_flat(p) ? p.flat_k[j] : p.ktab[t * p.n_cf + j]; }
__device__ __forceinline__ int64_t seg_koff(const Params& p, int t) { return is_flat(p) ? 0 : p.segs[t].koff; }
__device__ __forceinline__ int tile_seg(const Params& p, uint32_t u) { return is_flat(p) ? 0 : (int)p.tseg[u]; }
__device__ __forceinline__ bool seg_small(const Params& p, int t) { return !is_flat(p) && p.segs[t].small != 0u; }
// Copy blocks: one holds a copy of a (segment, CF)'s bracket histogram (NBIN words of hist1), a gather list (LCAP
// slots of list_*) and its fill count (a cache line of list_cnt).  Copy r of (t, j) is block seg_block(p, t, j) + r.
__device__ __forceinline__ uint32_t seg_rep(const Params& p, int t) { return is_flat(p) ? (uint32_t)REP : p.segs[t].rep; }
__device__ __forceinline__ size_t seg_block(const Params& p, int t, int j)
{
    return is_flat(p) ? (size_t)j * REP : (size_t)p.segs[t].pool0 + (size_t)j * p.segs[t].rep;
}

__device__ __forceinline__ uint32_t key_of(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

// Bin of the sample histogram a key falls into, and the keys a bin spans.
__device__ __forceinline__ uint32_t sample_bin(uint32_t key)
{
    if (key < SKEY0) return 0u;
    const uint32_t b = (key - SKEY0) >> SSHIFT;
    return b < (uint32_t)SBIN - 1u ? b : (uint32_t)SBIN - 1u;
}
__device__ __forceinline__ uint32_t sample_bin_first(uint32_t b) { return b == 0u ? 0u : SKEY0 + (b << SSHIFT); }
__device__ __forceinline__ uint32_t sample_bin_end(uint32_t b)
{
    return b == (uint32_t)SBIN - 1u ? KEY_END : SKEY0 + ((b + 1u) << SSHIFT);
}

// The bracket histogram of a CF whose bracket is [lo, hi): the shift s is the smallest with which bins 0 .. OVF - 1
// reach hi, and top is the first key past them (KEY_END if they reach past the largest key).
__device__ __forceinline__ void bracket_bins(uint32_t lo, uint32_t hi, uint32_t& s, uint32_t& top)
{
    const uint32_t span = hi > lo ? hi - lo : 0u;
    s = 0;
    if (span == 0u) { top = lo; return; }  // an empty bracket: every key from lo on counts as above it
    while ((span >> s) > OVF - 1u) ++s;
    const uint64_t t = (uint64_t)lo + ((uint64_t)OVF << s);
    top = t >= (uint64_t)KEY_END ? KEY_END : (uint32_t)t;
}

// Random-k: priority of index i, a keyed bijection of the 31-bit integers (adding a constant, multiplying
// by an odd constant and xor with a right shift are all bijections of [0, 2^31)), so no two indices tie.
__device__ __forceinline__ uint32_t priority_of(uint32_t s0, uint32_t s1, uint32_t i)
{
    const uint32_t M = 0x7FFFFFFFu;
    uint32_t x = (i + s0) & M;
    x ^= x >> 16; x = (x * 0x7FEB352Du) & M;
    x ^= x >> 15; x = (x * 0x046CA68Bu) & M;
    x ^= x >> 16; x = (x + s1) & M;
    x ^= x >> 14; x = (x * 0x2C1B3C6Du) & M;
    x ^= x >> 15; x = (x * 0x297A2D39u) & M;
    x ^= x >> 15;
    return x;
}

// The ordering key of a candidate: from its value (Top-k) or from its index (Random-k).
__device__ __forceinline__ uint32_t cand_key(const Params& p, int32_t idx, float val)
{
    return p.random ? priority_of(p.rk_s0, p.rk_s1, (uint32_t)idx) : key_of(val);
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Cross-lane sums with DPP (data-parallel primitives of the vector ALU) instead of LDS permutes: a step costs an
// instruction, not a round trip through the LDS crossbar, which matters where a wavefront's reductions sit on the
// critical path of a short kernel.  A row is 16 lanes; a lane whose source does not exist reads 0.
constexpr int DPP_QUAD_1032 = 0xB1, DPP_QUAD_2301 = 0x4E;       // quad_perm:[1,0,3,2], quad_perm:[2,3,0,1]
constexpr int DPP_ROW_SHR = 0x110, DPP_ROW_ROR = 0x120;         // + n: row_shr:n, row_ror:n
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143; // lane 15 of a row to the next row; lane 31 to rows 2 and 3

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ double dpp_move(double v)
{
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = dpp_move<CTRL, ROW_MASK>((uint32_t)b), hi = dpp_move<CTRL, ROW_MASK>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));   // a missing source gives +0.0
}

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint64_t dpp_move(uint64_t v)
{
    const uint32_t lo = dpp_move<CTRL, ROW_MASK>((uint32_t)v), hi = dpp_move<CTRL, ROW_MASK>((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t last_lane(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, 63); }
__device__ __forceinline__ uint64_t last_lane(uint64_t v)
{
    return ((uint64_t)last_lane((uint32_t)(v >> 32)) << 32) | last_lane((uint32_t)v);
}
__device__ __forceinline__ double last_lane(double v)
{
    return __longlong_as_double((long long)last_lane((uint64_t)__double_as_longlong(v)));
}

// Sum over the 64 lanes, the same value (and for floating point the same order of additions) in every lane:
// pairs, quads, the row's four quads, then rows 0+1 and 2+3, then all in lane 63, which is broadcast.
template <typename T>
__device__ __forceinline__ T wave_sum_t(T v)
{
    v += dpp_move<DPP_QUAD_1032>(v);
    v += dpp_move<DPP_QUAD_2301>(v);
    v += dpp_move<DPP_ROW_ROR + 4>(v);
    v += dpp_move<DPP_ROW_ROR + 8>(v);
    v += dpp_move<DPP_ROW_BCAST15, 0xA>(v);
    v += dpp_move<DPP_ROW_BCAST31, 0xC>(v);
    return last_lane(v);
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { return wave_sum_t(v); }
__device__ __forceinline__ double wave_sum(double v) { return wave_sum_t(v); }
__device__ __forceinline__ uint64_t wave_sum(uint64_t v) { return wave_sum_t(v); }

__device__ __forceinline__ double wave_max(double v)
{
    v = fmax(v, dpp_move<DPP_QUAD_1032>(v));   // (the values are not negative: a missing source's +0.0 changes nothing)
    v = fmax(v, dpp_move<DPP_QUAD_2301>(v));
    v = fmax(v, dpp_move<DPP_ROW_ROR + 4>(v));
    v = fmax(v, dpp_move<DPP_ROW_ROR + 8>(v));
    v = fmax(v, dpp_move<DPP_ROW_BCAST15, 0xA>(v));
    v = fmax(v, dpp_move<DPP_ROW_BCAST31, 0xC>(v));
    return last_lane(v);
}

// inclusive prefix sum over the lanes of a wavefront: within the rows first, then the earlier rows' totals
__device__ __forceinline__ uint32_t wave_scan(uint32_t v)
{
    uint32_t s = v + dpp_move<DPP_ROW_SHR + 1>(v);
    s += dpp_move<DPP_ROW_SHR + 2>(v);
    s += dpp_move<DPP_ROW_SHR + 3>(v);
    s += dpp_move<DPP_ROW_SHR + 4>(s);
    s += dpp_move<DPP_ROW_SHR + 8>(s);
    s += dpp_move<DPP_ROW_BCAST15, 0xA>(s);
    s += dpp_move<DPP_ROW_BCAST31, 0xC>(s);
    return s;
}

__device__ __forceinline__ uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// The entries of a tile's lists are the concatenation of its SUB sub-tile lists.
struct TileLists {
    uint32_t start[SUB + 1];  // start[j] = entries in sub-tiles before j; start[SUB] = all
    __device__ __forceinline__ uint32_t total() const { return start[SUB]; }
    // slot (relative to the tile's first slot) of the tile's i-th entry
    __device__ __forceinline__ uint32_t slot(uint32_t i) const
    {
        uint32_t j = 0;
#pragma unroll
        for (int x = 1; x < SUB; ++x) j += (i >= start[x]);
        uint32_t s = 0;
#pragma unroll
        for (int x = 1; x < SUB; ++x) if ((uint32_t)x == j) s = start[x];
        return j * TS + (i - s);
    }
};

// from the per-sub-tile counts cnt[u * SUB ..]; a count's DENSE_BIT is masked off (such a sub-tile lists nothing)
__device__ __forceinline__ TileLists tile_lists(const uint32_t* cnt, uint32_t u)
{
    TileLists c;
    c.start[0] = 0;
#pragma unroll
    for (int j = 0; j < SUB; ++j) {
        const uint32_t x = cnt[(size_t)u * SUB + j];
        c.start[j + 1] = c.start[j] + ((x & DENSE_BIT) ? 0u : x);
    }
    return c;
}

// The entries of a tile that the steps after the pass over the gradient look at one by one: all that lie inside
// some CF's bracket.  They are the sub-tile's bracket list, or, where the committed CF is the lowest of the call and
// the sub-tile keeps a candidate list, that list (which then holds them all, next to entries above the brackets).
struct TileRef {
    TileLists tl;        // such entries per sub-tile
    uint32_t main_mask;  // bit j: sub-tile j's are its candidate list
};

__device__ __forceinline__ TileRef tile_ref(const Params& p, uint32_t u)
{
    TileRef r;
    r.tl.start[0] = 0;
    r.main_mask = 0;
#pragma unroll
    for (int j = 0; j < SUB; ++j) {
        const uint32_t cc = p.cand_cnt[(size_t)u * SUB + j], bc = p.brk_cnt[(size_t)u * SUB + j];
        const bool use_main = !p.split && !(cc & DENSE_BIT);
        if (use_main) r.main_mask |= 1u << j;
        r.tl.start[j + 1] = r.tl.start[j] + (use_main ? cc : bc);
    }
    return r;
}

// Key (and value: needed for Random-k only, else 0) of the tile's i-th such entry, i < r.tl.total().
__device__ __forceinline__ void ref_entry(const Params& p, uint32_t u, const TileRef& r, uint32_t i, uint32_t& key, float& val)
{
    const uint32_t sl = r.tl.slot(i);
    const bool from_main = (r.main_mask >> (sl / TS)) & 1u;
    const size_t at = (size_t)u * TW + sl;
    if (!p.random) {
        // the bits of |acc| either way: a candidate's value with its sign, or the key itself
        const uint32_t* src = from_main ? (const uint32_t*)p.cand_val : p.brk_key;
        key = src[at] & 0x7FFFFFFFu;
        val = 0.0f;
    } else if (from_main) {
        key = priority_of(p.rk_s0, p.rk_s1, (uint32_t)p.cand_idx[at]);
        val = p.cand_val[at];
    } else {
        key = p.brk_key[at];
        val = p.brk_val[at];
    }
}


// One wavefront finds the bin of a 2048-bin histogram (given as `copies` arrays of NBIN counts that
// are added up) that holds the k-th largest entry: scanning from the top bin down,
// above < k <= above + count.  Every lane gets the result; bin == NONE if the histogram holds
// fewer than k entries.  hist must be 16-byte aligned.  Two passes, so that no lane has to keep its 32 bins
// in registers (this runs inside kernels whose occupancy matters): first the lane totals, which single out the
// lane whose bins hold the crossing, then that lane's 32 bins, one per lane.
__device__ __forceinline__ void wave_locate_bin(const uint32_t* hist, int copies, const uint32_t* top_extra, uint32_t k,
                                                uint32_t& bin, uint32_t& above, uint32_t& count)
{
    const int lane = threadIdx.x & 63;
    // top_extra: 64 more counts for the last bin, one per cache line (stride 32 words), or null
    const uint32_t extra = wave_sum(top_extra ? top_extra[lane * 32] : 0u);
    uint32_t mine = 0;  // lane l owns bins 32 l .. 32 l + 31
    for (int r = 0; r < copies; ++r) {
        const uint4* hv = (const uint4*)(hist + (size_t)r * NBIN + 32 * lane);
#pragma unroll 2
        for (int q = 0; q < 8; ++q) {
            const uint4 v = hv[q];
            mine += v.x + v.y + v.z + v.w;
        }
    }
    if (lane == 63) mine += extra;
    const uint32_t incl = wave_scan(mine);
    const uint32_t total = __shfl(incl, 63, 64);
    const uint32_t ab = total - incl;  // entries in the bins of higher lanes
    const uint64_t m = __ballot(ab < k && ab + mine >= k);
    if (m == 0ull) { bin = NONE; above = 0; count = 0; return; }
    const int owner = __ffsll((unsigned long long)m) - 1;
    const uint32_t ab_owner = __shfl(ab, owner, 64);
    // lanes 0..31 each take one of the owner's bins
    uint32_t c = 0;
    if (lane < 32) {
        for (int r = 0; r < copies; ++r) c += hist[(size_t)r * NBIN + 32 * owner + lane];
        if (owner == 63 && lane == 31) c += extra;
    }
    // entries of the owner's bins above bin `lane`: suffix sum over lanes lane+1 .. 31
    const uint32_t inc = wave_scan(c);                       // lanes >= 32 contribute 0
    const uint32_t sum32 = __shfl(inc, 31, 64);
    const uint32_t higher = ab_owner + (sum32 - inc);
    const uint64_t f = __ballot(lane < 32 && higher < k && higher + c >= k);
    const int src = 63 - __builtin_clzll((unsigned long long)f);  // exactly one lane
    bin = 32 * owner + src;
    above = __shfl(higher, src, 64);
    count = __shfl(c, src, 64);
}

// The same search by four wavefronts (threads q = 0..255 of a 256-thread team; `q` is the thread's number
// inside the team, `scratch` 8 words of LDS owned by the team).  Thread q owns bins 8q .. 8q+7 and has all
// its loads in flight at once.  The caller synchronises the team (all its threads reach this call) and
// provides the barrier: `sync()` must be a barrier that covers at least the team.
template <typename Sync>
__device__ __forceinline__ void team_locate_bin(const uint32_t* hist, int copies, const uint32_t* top_extra, uint32_t k,
                                                int q, uint32_t* scratch, Sync sync, uint32_t& bin, uint32_t& above,
                                                uint32_t& count)
{
    const int lane = q & 63, wv = q >> 6;
    uint32_t extra = (top_extra && q < 64) ? top_extra[q * 32] : 0u;
    uint32_t h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = 0;
    if (copies == REP) {
        uint4 v[REP][2];
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            const uint4* hv = (const uint4*)(hist + (size_t)r * NBIN + 8 * q);
            v[r][0] = hv[0]; v[r][1] = hv[1];
        }
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            h[0] += v[r][0].x; h[1] += v[r][0].y; h[2] += v[r][0].z; h[3] += v[r][0].w;
            h[4] += v[r][1].x; h[5] += v[r][1].y; h[6] += v[r][1].z; h[7] += v[r][1].w;
        }
    } else {
        for (int r = 0; r < copies; ++r) {
            const uint4* hv = (const uint4*)(hist + (size_t)r * NBIN + 8 * q);
            const uint4 a = hv[0], b = hv[1];
            h[0] += a.x; h[1] += a.y; h[2] += a.z; h[3] += a.w;
            h[4] += b.x; h[5] += b.y; h[6] += b.z; h[7] += b.w;
        }
    }
    extra = wave_sum(extra);  // non-zero in the team's first wavefront only
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) mine += h[i];
    const uint32_t incl = wave_scan(mine);
    if (lane == 63) scratch[wv] = incl;
    if (q == 0) scratch[4] = extra;
    sync();
    const uint32_t ex = scratch[4];  // belongs to the very last bin
    uint32_t total = ex, before = 0;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        total += scratch[x];
        if (x < wv) before += scratch[x];
    }
    uint32_t ab = total - ex - (before + incl);  // entries in the bins above this thread's eight ...
    if (q == 255) h[7] += ex;
    else ab += ex;                               // ... including the extra counts of the last bin
    uint32_t fb = NONE, fa = 0, fc = 0;
#pragma unroll
    for (int i = 7; i >= 0; --i) {
        if (ab < k && ab + h[i] >= k) { fb = 8 * q + i; fa = ab; fc = h[i]; }
        ab += h[i];
    }
    sync();  // scratch is rewritten below
    if (fb != NONE) { scratch[5] = fb; scratch[6] = fa; scratch[7] = fc; }
    if (q == 0) scratch[4] = (total >= k) ? 1u : 0u;
    sync();
    if (scratch[4]) { bin = scratch[5]; above = scratch[6]; count = scratch[7]; }
    else { bin = NONE; above = 0; count = 0; }
    sync();
}

// ---------------------------------------------------------------------------------------------
// S: layerwise mode, a tensor of at most SMALL_MAX elements: ONE workgroup does the whole step for it
// (error feedback, exact selection for every CF, statistics, message, residual) out of LDS, with no
// sample, no histogram in memory and no tile bookkeeping.  Its place in the message is known on the
// host (k_t is a function of the tensor's size), so nothing waits for it.  Runs as extra workgroups of
// the threshold kernel's launch (the workgroups that would otherwise have nothing to do for such a tensor).
// ---------------------------------------------------------------------------------------------
constexpr int SMALL_MAX = TW;              // elements
constexpr int SM_T = 1024;                 // threads
constexpr int SM_W = SM_T / 64;
constexpr int SM_PER = SMALL_MAX / SM_T;   // consecutive elements per thread
static_assert(SM_PER == 8, "see small_at");

struct SmallShared {
    float a[SMALL_MAX + SMALL_MAX / 32];   // acc, element i at i + i / 32: the runs of eight of 32 neighbouring threads
                                           // then fall into different banks
    uint32_t hist[256];
    uint32_t wg[SM_W], we[SM_W];
    uint32_t pick[2];
    uint32_t tau[MAXCF], need[MAXCF];      // per CF, kept by thread 0 for the statistics
    double ds[MAXCF + 1][SM_W];
};

__device__ __forceinline__ int small_at(int i) { return i + (i >> 5); }

__device__ __forceinline__ void small_segment(const Params& p, int t, SmallShared& sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    const int64_t s0 = p.segs[t].begin;
    const int nt = (int)(p.segs[t].end - s0);
    const int64_t koff = p.segs[t].koff;
    // acc into LDS, coalesced: all loads first and without branches around them (an element past the end reads the
    // last one instead and is not stored), so that they are in flight together
    {
        float gv[SM_PER], rv[SM_PER];
#pragma unroll
        for (int q = 0; q < SM_PER; ++q) {
            const int i = q * SM_T + tid;
            gv[q] = p.grad[s0 + (i < nt ? i : nt - 1)];
            rv[q] = 0.0f;
        }
        if (!p.single) {
#pragma unroll
            for (int q = 0; q < SM_PER; ++q) {
                const int i = q * SM_T + tid;
                rv[q] = p.res[s0 + (i < nt ? i : nt - 1)];
            }
        }
#pragma unroll
        for (int q = 0; q < SM_PER; ++q) {
            const int i = q * SM_T + tid;
            if (i < nt) sh.a[small_at(i)] = p.single ? gv[q] : rv[q] + gv[q];
        }
    }
    __syncthreads();
    // this thread's run: elements SM_PER tid .. SM_PER tid + nv - 1
    const int first = SM_PER * tid;
    const int nv = nt - first < 0 ? 0 : (nt - first > SM_PER ? SM_PER : nt - first);
    // (the keys stay in registers; the values are read from LDS again where they are needed)
    uint32_t key[SM_PER];
    double ssd = 0.0;
#pragma unroll
    for (int e = 0; e < SM_PER; ++e) {
        const float v = e < nv ? sh.a[small_at(first + e)] : 0.0f;
        key[e] = p.random ? priority_of(p.rk_s0, p.rk_s1, (uint32_t)(s0 + first + e)) : key_of(v);
        const double d = (double)v;
        ssd += d * d;
    }
    {
        const double w = wave_sum(ssd);
        if (lane == 0) sh.ds[MAXCF][wib] = w;
    }
    uint32_t tau_c = 0, need_c = 0;
    for (int j = 0; j < p.n_cf; ++j) {
        // the k-th largest key by four passes over the key's digits (8, 8, 8 and 7 bits from the top), each a
        // 256-bin histogram of the keys that agree with the digits found so far
        uint32_t want = p.ktab[(size_t)t * p.n_cf + j];
        uint32_t prefix = 0, mask = 0;
#pragma unroll 1
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = pass == 0 ? 23 : pass == 1 ? 15 : pass == 2 ? 7 : 0;
            const uint32_t dm = pass == 3 ? 127u : 255u;
            if (tid < 256) sh.hist[tid] = 0;
            __syncthreads();
            // (magnitudes crowd into a few digit values: a thread adds runs of equal digits at once)
            uint32_t cur = NONE, run = 0;
#pragma unroll
            for (int e = 0; e < SM_PER; ++e) {
                if (e < nv && (key[e] & mask) == prefix) {
                    const uint32_t dg = (key[e] >> shift) & dm;
                    if (dg != cur) {
                        if (run) atomicAdd(&sh.hist[cur], run);
                        cur = dg; run = 0;
                    }
                    ++run;
                }
            }
            if (run) atomicAdd(&sh.hist[cur], run);
            __syncthreads();
            if (wib == 0) {
                // lane l owns digits 4 l .. 4 l + 3; from the top: above < want <= above + count
                const uint32_t h0 = sh.hist[4 * lane], h1 = sh.hist[4 * lane + 1], h2 = sh.hist[4 * lane + 2], h3 = sh.hist[4 * lane + 3];
                const uint32_t mine = h0 + h1 + h2 + h3;
                const uint32_t incl = wave_scan(mine);
                const uint32_t total = __shfl(incl, 63, 64);
                uint32_t ab = total - incl;
                const uint32_t hh[4] = {h0, h1, h2, h3};
#pragma unroll
                for (int q = 3; q >= 0; --q) {
                    if (ab < want && ab + hh[q] >= want) { sh.pick[0] = 4u * lane + q; sh.pick[1] = ab; }
                    ab += hh[q];
                }
            }
            __syncthreads();
            prefix |= sh.pick[0] << shift;
            mask |= dm << shift;
            want -= sh.pick[1];
        }
        if (tid == 0) { sh.tau[j] = prefix; sh.need[j] = want; }   // want: the keys equal to tau that are selected
        if (j == p.commit) { tau_c = prefix; need_c = want; }
        // energy above the threshold (Random-k: and of the entry at it, which has no particular magnitude)
        double s = 0.0;
#pragma unroll
        for (int e = 0; e < SM_PER; ++e) {
            if (e < nv && (key[e] > prefix || (p.random && key[e] == prefix))) {
                const double d = (double)sh.a[small_at(first + e)];
                s += d * d;
            }
        }
        s = wave_sum(s);
        if (lane == 0) sh.ds[j][wib] = s;
    }
    // the committed CF's selection, in index order: a thread's run is consecutive, so the counts of the threads
    // before it give its place
    uint32_t g = 0, eq = 0;
#pragma unroll
    for (int e = 0; e < SM_PER; ++e) {
        g += (e < nv && key[e] > tau_c);
        eq += (e < nv && key[e] == tau_c);
    }
    const uint32_t ig = wave_scan(g), ie = wave_scan(eq);
    if (lane == 63) { sh.wg[wib] = ig; sh.we[wib] = ie; }
    __syncthreads();
    uint32_t run_g = ig - g, run_e = ie - eq;
#pragma unroll
    for (int w = 0; w < SM_W; ++w)
        if (w < wib) { run_g += sh.wg[w]; run_e += sh.we[w]; }
    const uint32_t ties_before = run_e < need_c ? run_e : need_c;
    int64_t o = koff + run_g + ties_before;
    const int64_t lim = koff + (int64_t)p.ktab[(size_t)t * p.n_cf + p.commit];
    uint32_t left = need_c - ties_before;
#pragma unroll
    for (int e = 0; e < SM_PER; ++e) {
        if (e >= nv) continue;
        bool sel = key[e] > tau_c;
        if (key[e] == tau_c && left > 0) { sel = true; --left; }
        if (sel) {
            if (o < lim) {   // (always, if the counts are consistent; never write out of range)
                p.out_val[o] = sh.a[small_at(first + e)];
                p.out_idx[o] = p.single ? p.map_idx[s0 + first + e] : (int32_t)(s0 + first + e);
            }
            ++o;
            if (!p.no_commit) sh.a[small_at(first + e)] = 0.0f;
        }
    }
    if (tid == 0) {
        // statistics: every wavefront's sums in order
        double ss_dense = 0.0;
        for (int w = 0; w < SM_W; ++w) ss_dense += sh.ds[MAXCF][w];
        for (int j = 0; j < p.n_cf; ++j) {
            double s = 0.0;
            for (int w = 0; w < SM_W; ++w) s += sh.ds[j][w];
            const double tauv = p.random ? (double)sh.tau[j] : (double)__uint_as_float(sh.tau[j]);
            if (!p.random) s += (double)sh.need[j] * tauv * tauv;
            double* os = p.out_stats + ((size_t)t * p.n_cf + j) * GRAVAC_STATS_PER_CF;
            os[0] = s;
            os[1] = ss_dense;
            os[2] = (ss_dense == 0.0) ? 1.0 : s / ss_dense;
            os[3] = tauv;
        }
    }
    __syncthreads();
    // the new residual (acc with the selection zeroed), coalesced; single-source mode: into the dense residual
#pragma unroll 4
    for (int q = 0; q < SM_PER; ++q) {
        const int i = q * SM_T + tid;
        if (i >= nt) continue;
        const float r = sh.a[small_at(i)];
        if (!p.single) {
            p.res[s0 + i] = r;
        } else if (p.restore) {
            const int mi = p.map_idx[s0 + i];
            if ((uint64_t)(int64_t)mi < (uint64_t)p.n_restore) p.restore[mi] = r;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// K0a: sample acc = residual + grad at stratified positions; each workgroup histograms its samples in
// LDS (SBIN bins of 2^17 keys, see sample_bin) and stores the counts as 16-bit numbers, and the
// counts per group of SBIN / SGRP bins beside them.  The same launch clears what the later kernels
// add to (every workgroup a share of its segment's histograms and counters); a call whose brackets
// do not come from a sample launches it for that alone.
// ---------------------------------------------------------------------------------------------
template <int R>  // R groups per thread: a workgroup histograms R * SAMPLE_BLOCK samples
__global__ __launch_bounds__(256) void sample_kernel(Params p)
{
    __shared__ uint32_t h[SBIN];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const int t = is_flat(p) ? 0 : (int)p.sblock_seg[b];
    const uint32_t lb = b - (is_flat(p) ? 0u : p.segs[t].samp0);
    const uint32_t S = is_flat(p) ? p.flat_samples : p.segs[t].samp_cnt;
    {
        // the segment's sample blocks share the clearing: block lb of nbk takes every nbk-th 16-byte piece
        const uint32_t per = SAMPLE_BLOCK * R;
        const uint32_t nbk = is_flat(p) ? p.n_sample_blocks : (S + per - 1) / per;
        const uint4 z = make_uint4(0u, 0u, 0u, 0u);
        const uint32_t blocks = (uint32_t)p.n_cf * seg_rep(p, t);  // the segment's copy blocks
        uint4* h1 = (uint4*)(p.hist1 + seg_block(p, t, 0) * NBIN);
        for (uint32_t i = lb * 256 + tid; i < blocks * NBIN / 4; i += nbk * 256) h1[i] = z;
        uint4* cs = (uint4*)(p.coarse + (size_t)t * NBIN);
        for (uint32_t i = lb * 256 + tid; i < NBIN / 4; i += nbk * 256) cs[i] = z;
        for (uint32_t i = lb * 256 + tid; i < (uint32_t)p.n_cf * 64; i += nbk * 256) p.ovfc[((size_t)t * p.n_cf * 64 + i) * 32] = 0;
        for (uint32_t i = lb * 256 + tid; i < blocks; i += nbk * 256) p.list_cnt[(seg_block(p, t, 0) + i) * 32] = 0;
    }
    if (p.bounds_from != BOUNDS_SAMPLED) return;
    const int64_t s0 = seg_begin(p, t);
    const uint64_t nt = (uint64_t)(seg_end(p, t) - s0);
#pragma unroll
    for (int q = 0; q < SBIN / 256; ++q) h[q * 256 + tid] = 0;
    __syncthreads();
    // A group is 4 consecutive elements: sample i of the segment is element i % 4 of group i / 4.  A sampled
    // segment (S a multiple of SAMPLE_BLOCK, nt > 2 S) is cut into S / 16 strata of at least 32 elements, and the
    // four groups of a stratum are the 16 elements of one line at a hashed place inside it: a sample costs a
    // sixteenth of the memory transactions that single elements at scattered places would (the sampling pass is
    // bound by their number, not by their bytes).
    static_assert(SAMPLE_BLOCK / 256 == 4, "groups of four");
    constexpr int Q = 4 * R;
    uint64_t gpos[R];
    bool live[Q];
    // stratum g16 of G = S / 16 spans [g16 nt / G, (g16 + 1) nt / G): with nt = G qd + rm that is g16 qd + g16 rm / G, one
    // 64-bit division per thread and 32-bit ones per stratum (g16 rm < G^2 <= 2^30) instead of 64-bit ones throughout
    const uint32_t G = S / 16 ? S / 16 : 1u;
    const uint64_t qd = nt / G;
    const uint32_t rm = (uint32_t)(nt - qd * G);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t g = (lb * R + r) * (SAMPLE_BLOCK / 4) + tid;  // group
        gpos[r] = 4ull * g;                                          // the whole segment is read: elements 4g .. 4g+3
        if ((uint64_t)S != nt) {
            // four neighbouring threads share one stratum and one run of 16 elements in it that starts at a multiple
            // of 16 in the flat buffer (a 64-byte line if the buffer is aligned to that)
            const uint32_t g16 = g >> 2;
            const uint64_t a = (uint64_t)g16 * qd + (g16 * rm) / G, e = (uint64_t)(g16 + 1) * qd + ((g16 + 1) * rm) / G;  // e - a >= 32
            const uint64_t first = ((uint64_t)s0 + a + 15) & ~15ull;                 // first such run inside the stratum
            const uint32_t runs = (uint32_t)(((uint64_t)s0 + e - first) / 16);        // >= 1
            const uint64_t at = first + 16ull * (hash32(g16 * 0x9E3779B9u + 0x85EBCA6Bu) % runs);
            gpos[r] = (at - (uint64_t)s0) + 4u * (g & 3u);                            // gpos + 3 < e <= nt
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) live[4 * r + q] = 4ull * g + q < S;
    }
    // all loads first, without branches around them (a group past the segment's last sample reads the segment's
    // last element instead and is not counted), so that they are in flight together
    float gv[Q], rv[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const uint64_t pos = gpos[q / 4] + (q & 3) < nt ? gpos[q / 4] + (q & 3) : nt - 1;
        gv[q] = p.grad[s0 + (int64_t)pos];
        rv[q] = 0.0f;
    }
    if (!p.single) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const uint64_t pos = gpos[q / 4] + (q & 3) < nt ? gpos[q / 4] + (q & 3) : nt - 1;
            rv[q] = p.res[s0 + (int64_t)pos];
        }
    }
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const float acc = p.single ? gv[q] : rv[q] + gv[q];
        if (live[q]) atomicAdd(&h[sample_bin(key_of(acc))], 1u);
    }
    __syncthreads();
    // thread i stores bins 16i .. 16i+15, two counts per word (a count is at most R * SAMPLE_BLOCK < 2^16)
    static_assert(R * SAMPLE_BLOCK < 65536, "16-bit counts");
    uint4 w[2];
    uint32_t* wp = (uint32_t*)w;
    uint32_t mine = 0;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        const uint32_t c0 = h[16 * tid + 2 * m], c1 = h[16 * tid + 2 * m + 1];
        wp[m] = c0 | (c1 << 16);
        mine += c0 + c1;
    }
    uint4* dst = (uint4*)(p.samp_hist + (size_t)b * (SBIN / 2) + 8 * tid);
    dst[0] = w[0];
    dst[1] = w[1];
    // a group of SBIN / SGRP = 512 bins is what 32 neighbouring threads hold: half a wavefront
    static_assert(SBIN / SGRP == 32 * 16 && SGRP == 8, "one group per half wavefront");
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
    if ((tid & 31) == 0) p.samp_grp[(size_t)b * SGRP + (tid >> 5)] = mine;
}

// ---------------------------------------------------------------------------------------------
// K0b: per segment, add up the sample histograms and turn the sampled ranks into a bracket of keys per
// CF.  G workgroups per segment; workgroup y adds up the bins [y, y + 1) * SBIN / G of all the
// segment's sample blocks (what lies above them it knows from the blocks' group counts) and writes the
// bracket ends that fall into its bins, so that no workgroup waits for another.  The kernels that
// use the brackets derive the histogram shift and the rest from them (bracket_bins).
// ---------------------------------------------------------------------------------------------
// (the form with the small tensors is held to 64 registers, so that two of its 1024-thread workgroups fit a CU: a
// layerwise call has more such workgroups than the chip has CUs)
template <int G, bool SMALL, int P = 1>  // SMALL: the workgroups of tensors of at most SMALL_MAX elements do the whole step for them
__global__ __launch_bounds__(P * 1024 / G) __attribute__((amdgpu_waves_per_eu(SMALL ? 8 : 1, 8))) void threshold_kernel(Params p)
{
    constexpr int T = 1024 / G;          // thread i < T owns the bins 4 (y T + i) .. + 3: two words of every block's histogram
    // P threads per such set of bins: thread i + x T adds up the blocks x, x + P, ... (the 64 to 128 blocks of a flat
    // sample are then one round of loads per thread, not two to four; two threads are best up to 64 blocks, four beyond)
    static_assert(P * 1024 / G <= 1024 && (G > 1 || P == 1), "threads of a workgroup");
    constexpr int NW = T / 64;
    static_assert(G == 1 || G == SGRP, "one workgroup per group of bins, or one for all");
    __shared__ uint32_t wtot[NW], gab[NW], gto[NW];
    __shared__ uint32_t rank_lo[MAXCF], rank_hi[MAXCF], rank_mid[MAXCF];
    __shared__ uint32_t hx[P > 1 ? P - 1 : 1][P > 1 ? T : 1][4];
    const int t = blockIdx.x, y = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    const int part = tid / T, ot = tid - part * T;
    if (t == 0 && y == 0 && tid == 0) {
        p.status->any_fail = 0; p.status->n_fail = 0; p.status->error = 0; p.status->n_seg = p.n_seg;
        p.status->n_narrow = 0; p.status->count = 0;
        if (p.out_count && p.bounds_from != BOUNDS_FIXED) *p.out_count = p.total_out;  // (else the scan knows it)
    }
    if constexpr (SMALL) {
        static_assert(G == 1 && SM_T == 1024, "the small tensors' workgroups are this kernel's");
        __shared__ SmallShared small;
        if (seg_small(p, t)) {
            small_segment(p, t, small);
            return;
        }
    }
    const uint32_t S = is_flat(p) ? p.flat_samples : p.segs[t].samp_cnt;
    const uint32_t sb0 = is_flat(p) ? 0u : p.segs[t].samp0;
    const uint32_t nb = is_flat(p) ? p.n_sample_blocks : (S + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
    const uint64_t nt = (uint64_t)(seg_end(p, t) - seg_begin(p, t));
    const bool whole = ((uint64_t)S == nt);
    const bool sampled = p.bounds_from == BOUNDS_SAMPLED;
    if (y == 0) {
        if (!is_flat(p))
            for (uint32_t u = seg_tile0(p, t) + tid; u < seg_tile1(p, t); u += T * P) p.tseg[u] = (uint32_t)t;
        if (tid == 0) p.seg[t].fail = FAIL_NONE;  // the locate step raises it
    }
    if (tid < p.n_cf) {
        const uint32_t k = seg_k(p, t, tid);
        uint32_t r_lo, r_hi, r_mid;
        if (whole) {
            r_lo = r_hi = r_mid = k;
        } else {
            // expected number of sampled keys among the k largest, widened by ZMARGIN standard deviations
            const double m = (double)k * (double)S / (double)nt, sd = sqrt(m);
            const double a = ceil(m + ZMARGIN * sd + 2.0), b = floor(m - ZMARGIN * sd - 2.0);
            r_lo = (a >= 4.0e9) ? NONE : (uint32_t)a;
            r_hi = (b < 1.0) ? 1u : (uint32_t)b;
            r_mid = (m < 1.0) ? 1u : (m >= 4.0e9 ? NONE : (uint32_t)(m + 0.5));
        }
        rank_lo[tid] = r_lo; rank_hi[tid] = r_hi; rank_mid[tid] = r_mid;
    }
    if (p.bounds_from == BOUNDS_FIXED) {
        // the threshold sparsifier (one flat tensor, one "CF"): an empty bracket at the caller's threshold, so that the
        // pass over the gradient counts and lists what lies at or above it; the later steps find everything resolved:
        // selected <=> key > tau with tau one key below the threshold, no ties to take
        if (tid == 0) {
            p.bnd_lo[0] = p.fixed_key; p.bnd_hi[0] = p.fixed_key; p.bnd_mid[0] = NONE;
            CfState st;
            st.k = 0; st.lo = p.fixed_key; st.s = 0; st.mode = MODE_RESOLVED; st.base = p.fixed_key; st.span = 0;
            st.above = 0; st.c = 0; st.tau = p.fixed_key - 1u; st.need = 0; st.cnt_gt = 0; st.redo = 0; st.lo2 = 0; st.s2 = 0;
            st.top = p.fixed_key; st.pad = 0;
            p.st[0] = st;
            SegState sg;
            sg.lo_min = p.fixed_key; sg.fail = FAIL_NONE; sg.pz = p.single ? NONE : p.fixed_key; sg.lo_c = p.fixed_key;
            p.seg[0] = sg;
        }
        return;
    }
    if (!sampled) {
        // no sample: the brackets follow from k alone (Random-k) or are left empty (every segment takes the exact route)
        if (y == 0 && tid < p.n_cf) {
            uint32_t lo = NONE, hi = NONE, mid = NONE;
            if (p.bounds_from == BOUNDS_RANDOM) {
                // priorities are a keyed permutation of the 31-bit integers: the number of a tensor's nt indices
                // with priority >= x is as good as binomial (nt, 1 - x / 2^31), so the bounds follow from k alone:
                // x with k + ZMARGIN sqrt(k) + 2 expected above it, and x with k - ZMARGIN sqrt(k) - 2
                const double k = (double)seg_k(p, t, tid), w = ZMARGIN * sqrt(k) + 2.0;
                const double q_lo = (k + w) / (double)nt, q_hi = (k - w) / (double)nt;
                lo = q_lo >= 1.0 ? 0u : (uint32_t)floor(2147483648.0 * (1.0 - q_lo));
                hi = q_hi <= 0.0 ? KEY_END : (uint32_t)ceil(2147483648.0 * (1.0 - q_hi));
                mid = (uint32_t)floor(2147483648.0 * (1.0 - (k >= (double)nt ? 1.0 : k / (double)nt)));
            }
            p.bnd_lo[(size_t)t * p.n_cf + tid] = lo;
            p.bnd_hi[(size_t)t * p.n_cf + tid] = hi;
            p.bnd_mid[(size_t)t * p.n_cf + tid] = mid;
        }
        return;
    }
    // samples in the groups of bins above this workgroup's, and in all
    // (the group counts of up to two blocks per thread are fetched first and added up after the histograms, so that
    // both sets of loads are in flight together)
    uint32_t g_above = 0, g_total = 0;
    uint4 ga[2][2];
    static_assert(G == 1 || 2 * (1024 / G) >= 2 * DENSE_BLOCKS, "two blocks' group counts per thread cover a flat sample");
    if (G > 1 && part == 0) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const uint32_t b = ot + x * T;
            const uint4* gp = (const uint4*)(p.samp_grp + (size_t)(sb0 + (b < nb ? b : 0u)) * SGRP);
            ga[x][0] = gp[0]; ga[x][1] = gp[1];
        }
    }
    uint32_t h0 = 0, h1 = 0, h2 = 0, h3 = 0;
    {
        const uint2* src = (const uint2*)(p.samp_hist + (size_t)sb0 * (SBIN / 2)) + (y * T + ot);
        constexpr int NB = SMALL ? 16 : 32;   // loads in flight per thread
        for (uint32_t b0 = (uint32_t)part; b0 < nb; b0 += NB * P) {
            uint2 w[NB];
#pragma unroll
            for (int q = 0; q < NB; ++q) w[q] = (b0 + q * P < nb) ? src[(size_t)(b0 + q * P) * (SBIN / 4)] : make_uint2(0u, 0u);
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                h0 += w[q].x & 0xFFFFu; h1 += w[q].x >> 16;
                h2 += w[q].y & 0xFFFFu; h3 += w[q].y >> 16;
            }
        }
    }
    if (P > 1) {
        if (part != 0) {
            uint32_t* d = hx[part - 1][ot];
            d[0] = h0; d[1] = h1; d[2] = h2; d[3] = h3;
            h0 = h1 = h2 = h3 = 0;
        }
        __syncthreads();
        if (part == 0) {
#pragma unroll
            for (int x = 0; x < P - 1; ++x) { h0 += hx[x][ot][0]; h1 += hx[x][ot][1]; h2 += hx[x][ot][2]; h3 += hx[x][ot][3]; }
        }
    }
    if (G > 1 && part == 0) {
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            if (ot + x * T >= nb) continue;
            const uint32_t v[8] = {ga[x][0].x, ga[x][0].y, ga[x][0].z, ga[x][0].w, ga[x][1].x, ga[x][1].y, ga[x][1].z, ga[x][1].w};
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                g_total += v[g];
                if (g > y) g_above += v[g];
            }
        }
        g_above = wave_sum(g_above);
        g_total = wave_sum(g_total);
        if (lane == 0) { gab[wib] = g_above; gto[wib] = g_total; }
    }
    const uint32_t mine = h0 + h1 + h2 + h3;
    const uint32_t incl = wave_scan(mine);
    if (lane == 63 && part == 0) wtot[wib] = incl;
    __syncthreads();
    if (part != 0) return;   // (no barrier follows)
    uint32_t local = 0, before = 0;
    g_above = 0; g_total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t x = wtot[w];
        local += x;
        if (w < wib) before += x;
        if (G > 1) { g_above += gab[w]; g_total += gto[w]; }
    }
    if (G == 1) g_total = local;
    const uint32_t above0 = g_above + local - (before + incl);  // samples in bins above this thread's four
    const uint32_t hh[4] = {h0, h1, h2, h3};
    for (int j = 0; j < p.n_cf; ++j) {
        const uint32_t r_lo = rank_lo[j], r_hi = rank_hi[j], r_mid = rank_mid[j];
        const size_t id = (size_t)t * p.n_cf + j;
        uint32_t above = above0;
#pragma unroll
        for (int q = 3; q >= 0; --q) {
            const uint32_t c = hh[q];
            const uint32_t bin = 4u * (uint32_t)(y * T + ot) + (uint32_t)q;
            // lower edge of the bin of the r_lo-th sample from the top, upper edge of the bin of the r_hi-th
            if (above < r_lo && above + c >= r_lo) p.bnd_lo[id] = sample_bin_first(bin);
            if (above < r_hi && above + c >= r_hi) p.bnd_hi[id] = sample_bin_end(bin);
            if (above < r_mid && above + c >= r_mid) {
                // the r_mid-th sample from the top is the (r_mid - above)-th of the c in this bin: that far down from
                // the bin's upper edge, as if the bin's samples were spread evenly over its keys
                const uint32_t first = sample_bin_first(bin), end = sample_bin_end(bin);
                // (an estimate: single precision will do, and keeps a 64-bit division out of this kernel)
                const uint32_t down = (uint32_t)((float)(end - first) * ((float)(r_mid - above) / (float)c));
                p.bnd_mid[id] = down >= end - first ? first : end - down;
            }
            above += c;
        }
        // fewer samples than a rank: the bracket is open on that side
        if (y == 0 && tid == 0) {
            if (g_total < r_lo) p.bnd_lo[id] = 0u;
            if (g_total < r_hi) p.bnd_hi[id] = KEY_END;
            if (g_total < r_mid) p.bnd_mid[id] = NONE;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// K1: the pass over the gradient, one sub-tile per wavefront.
//     SM_EF: read grad and residual, write acc back, sum acc^2.
//     SM_EXACT (exact route, failed segments only): read acc from residual; the brackets come from the
//     coarse histogram.  Both collect the lists of the sub-tile in index order.
// ---------------------------------------------------------------------------------------------
// From which key on the pass over the gradient stores +0 instead of acc in a sub-tile that lists its candidates
// (NONE: nowhere): the key the sample puts the committed CF's k-th largest at, kept inside that CF's bracket
// [lo, top).  Entries from there on are in the candidate list, and most of them are selected: the emit step then has
// a scattered store only for the entries between this key and the threshold, selected ones below it (+0) or
// unselected ones at or above it (acc put back), instead of one for every selected entry of the bracket; a
// scattered 4-byte store costs the memory a read and a write of its 64 bytes, 34 us per million of them.
__device__ __forceinline__ uint32_t zero_from(const Params& p, int t, uint32_t lo, uint32_t top)
{
    if (p.single || p.no_commit || top == KEY_END) return NONE;
    const uint32_t mid = p.bnd_mid[(size_t)t * p.n_cf + p.commit];
    if (mid == NONE) return top;
    return mid < lo ? lo : (mid > top ? top : mid);
}

template <int NCF>  // compiled for calls with up to NCF CFs: the loops over the CFs are unrolled
struct SubCtx {
    uint32_t lo_min, lo_c, pz;
    uint32_t lo[NCF];
    uint32_t sh[NCF];
    uint32_t top[NCF];
    uint32_t ovn[NCF];     // entries above CF j's bracket ...
    double ovs[NCF];       // ... and their sum of acc^2
    bool split;            // the entries inside the brackets get a list of their own in every sub-tile
    uint32_t* h1;   // this wavefront's copy of the bracket histograms of the tile's segment ...
    uint32_t hstride;  // ... whose CFs are this many words apart
    int32_t* cidx;  // candidate-list slots of this sub-tile
    float* cval;
    uint32_t run;   // candidates listed so far
    uint32_t* bkey; // bracket-list slots of this sub-tile
    float* bval;
    uint32_t brun;  // bracket entries listed so far
    double ssd;
    int ncf;
    uint32_t s0, s1;  // Random-k keys
};

// What one entry with key >= lo_min adds: per CF whose bracket starts at or below it, a count above the bracket or
// a histogram update inside it.  Returns whether it lies inside some CF's bracket.
template <int NCF>
__device__ __forceinline__ bool bracket_count(SubCtx<NCF>& c, uint32_t key, float a)
{
    bool inside = false;
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        if ((j == 0 || j < c.ncf) && key >= c.lo[j]) {
            if (key >= c.top[j]) {
                const double d = (double)a;
                c.ovn[j]++;
                c.ovs[j] += d * d;
            } else {
                atomicAdd(&c.h1[j * c.hstride + ((key - c.lo[j]) >> c.sh[j])], 1u);
                inside = true;
            }
        }
    }
    return inside;
}

__device__ __forceinline__ v4f ld_stream(const v4f* q)
{
#if GV_NT
    return __builtin_nontemporal_load(q);
#else
    return *q;
#endif
}

__device__ __forceinline__ void st_stream(v4f v, v4f* q)
{
#if GV_NT
    __builtin_nontemporal_store(v, q);
#else
    *q = v;
#endif
}

// The ordering keys of one lane's four consecutive elements a[0..3] at global index g.
template <bool RND, int NCF>
__device__ __forceinline__ void keys_of_row(const SubCtx<NCF>& c, const float a[4], int64_t g, uint32_t key[4])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) key[e] = RND ? priority_of(c.s0, c.s1, (uint32_t)(g + e)) : key_of(a[e]);
}

// One lane's four consecutive elements a[0..3] with keys key[0..3] at global index g; vm = validity bits;
// listed = whether the sub-tile keeps a candidate list (the same for all lanes).
template <bool SSD, bool RND, int NCF>
__device__ __forceinline__ void consume(SubCtx<NCF>& c, const float a[4], const uint32_t key[4], int64_t g, unsigned vm, bool listed)
{
    bool f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const bool valid = (vm >> e) & 1u;
        f[e] = valid && key[e] >= c.lo_min;
        if (SSD) {
            const double d = valid ? (double)a[e] : 0.0;
            c.ssd += d * d;
        }
    }
    if (__ballot(f[0] | f[1] | f[2] | f[3]) == 0ull) return;
    bool fb[4], fm[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        fb[e] = f[e] ? bracket_count(c, key[e], a[e]) : false;
        fm[e] = listed && f[e] && key[e] >= c.lo_c;
    }
    if (__ballot(fm[0] | fm[1] | fm[2] | fm[3]) != 0ull) {
        uint32_t pre = 0, tot = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t m = __ballot(fm[e]);
            pre += lanes_below(m);
            tot += (uint32_t)__popcll(m);
        }
        uint32_t w = c.run + pre;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (fm[e]) {
                c.cidx[w] = (int32_t)(g + e);
                c.cval[w] = a[e];
                ++w;
            }
        }
        c.run += tot;
    }
    // the entries inside the brackets: a list of their own, unless the candidate list holds them all
    if ((c.split || !listed) && __ballot(fb[0] | fb[1] | fb[2] | fb[3]) != 0ull) {
        uint32_t pre = 0, tot = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t m = __ballot(fb[e]);
            pre += lanes_below(m);
            tot += (uint32_t)__popcll(m);
        }
        uint32_t w = c.brun + pre;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (fb[e]) {
                c.bkey[w] = key[e];
                if (RND) c.bval[w] = a[e];
                ++w;
            }
        }
        c.brun += tot;
    }
}

// Modes of the pass.
enum { SM_EF = 0,      // acc = residual + grad, written back into residual
       SM_EXACT = 1,   // exact route: acc is re-read, the lists are collected again
       SM_SINGLE = 2   // single source (second-level compression): acc = grad; every value is also written
};                     // back into the dense residual at its mapped index (the emit pass zeroes the selected)

// Issue the loads of one row (this lane's four elements from global index g).
template <int M>
__device__ __forceinline__ void row_load(const Params& p, int64_t g, v4f& x, v4f& y, v4i& m)
{
    if (M == SM_EF) { x = ld_stream((const v4f*)(p.res + g)); y = ld_stream((const v4f*)(p.grad + g)); }
    if (M == SM_EXACT) x = ld_stream((const v4f*)(p.acc + g));
    if (M == SM_SINGLE) {
        y = ld_stream((const v4f*)(p.grad + g));
        if (p.restore) m = *(const v4i*)(p.map_idx + g);
    }
}

// Arithmetic of one row; a[] gets the four acc values.
template <int M>
__device__ __forceinline__ void row_finish(const Params& p, const v4f& x, const v4f& y, const v4i& m, float a[4])
{
    if (M == SM_EF) {
        const v4f av = x + y;  // stored once the keys are known
        a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
    }
    if (M == SM_EXACT) { a[0] = x.x; a[1] = x.y; a[2] = x.z; a[3] = x.w; }
    if (M == SM_SINGLE) {
        a[0] = y.x; a[1] = y.y; a[2] = y.z; a[3] = y.w;
        if (p.restore) {
            const int mi[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((uint64_t)(int64_t)mi[e] < (uint64_t)p.n_restore) p.restore[mi[e]] = a[e];
        }
    }
}

// One element of a row that is not handled with 16-byte accesses.
template <int M>
__device__ __forceinline__ float element_load(const Params& p, int64_t q)
{
    if (M == SM_EF) return p.res[q] + p.grad[q];
    if (M == SM_EXACT) return p.acc[q];
    const float a = p.grad[q];
    if (p.restore) {
        const int mi = p.map_idx[q];
        if ((uint64_t)(int64_t)mi < (uint64_t)p.n_restore) p.restore[mi] = a;
    }
    return a;
}

// Exact route: the bounds of the segment a wavefront last worked on (they cost a histogram search).
struct ExactBounds {
    int t;  // segment, -1 = none yet
    uint32_t lo[MAXCF];
    uint32_t sh[MAXCF];
    uint32_t top[MAXCF];   // narrow route: the end of the bracket the lists were collected with
    uint32_t end[MAXCF];   // first key past the XBINS bins
    uint32_t lo_min, lo_c;
};

// One sub-tile v, by one wavefront.
template <int M, bool RND, int NCF>
__device__ __forceinline__ void stream_subtile(const Params& p, uint32_t v, int lane, ExactBounds* xb)
{
    constexpr bool EF = (M != SM_EXACT);  // a first pass: sums acc^2, takes the brackets from the threshold kernel
    const uint32_t u = v / SUB;  // tile
    if (u >= p.n_tiles) return;
    const int t = tile_seg(p, u);
    const uint32_t fail_kind = EF ? (uint32_t)FAIL_NONE : p.seg[t].fail;
    if (!EF && fail_kind == FAIL_NONE) return;
    const int64_t sb = seg_begin(p, t), se = seg_end(p, t);
    const int64_t s0 = sb + (int64_t)(u - seg_tile0(p, t)) * TW + (int64_t)(v % SUB) * TS;
    const int64_t e0 = (s0 + TS < se) ? s0 + TS : se;
    const bool narrow = !EF && fail_kind == FAIL_NARROW;
    if (s0 >= se && !narrow) {  // sub-tile past the end of the segment
        if (lane == 0) { p.cand_cnt[v] = 0; p.brk_cnt[v] = 0; if (EF) p.ssd[v] = 0.0; }
        if (lane < p.n_cf) { p.ovn[(size_t)v * p.n_cf + lane] = 0; p.ovs[(size_t)v * p.n_cf + lane] = 0.0; }
        return;
    }

    SubCtx<NCF> c;
    c.ncf = p.n_cf;
    c.split = p.split != 0;
    c.s0 = p.rk_s0; c.s1 = p.rk_s1;
    c.lo_min = NONE; c.lo_c = NONE; c.pz = NONE;
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        c.ovn[j] = 0; c.ovs[j] = 0.0;
        c.lo[j] = NONE; c.sh[j] = 0; c.top[j] = KEY_END;
    }
    if (EF) {
#pragma unroll
        for (int j = 0; j < NCF; ++j) {
            if (j < p.n_cf) {
                c.lo[j] = p.bnd_lo[(size_t)t * p.n_cf + j];
                bracket_bins(c.lo[j], p.bnd_hi[(size_t)t * p.n_cf + j], c.sh[j], c.top[j]);
                c.lo_min = c.lo[j] < c.lo_min ? c.lo[j] : c.lo_min;
                if (j == p.commit) {
                    c.lo_c = c.lo[j];
                    if (M == SM_EF) c.pz = zero_from(p, t, c.lo[j], c.top[j]);
                }
            }
        }
        if (!c.split) c.lo_c = c.lo_min;  // the candidate list takes every entry that concerns some CF
    } else {
        const bool first = (v == seg_tile0(p, t) * SUB);
        if (xb->t != t) {
            xb->t = t;
            xb->lo_min = NONE; xb->lo_c = NONE;
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) {
                xb->lo[j] = NONE; xb->sh[j] = 10; xb->top[j] = KEY_END; xb->end[j] = KEY_END;
                if (j < p.n_cf) {
                    const CfState* st = &p.st[(size_t)t * p.n_cf + j];
                    if (narrow) {
                        // the locate step has left the bounds of the CFs that are binned again; the others keep
                        // their histogram and their plan (lo = NONE: no key is counted for them here)
                        if (st->redo) { xb->lo[j] = st->lo2; xb->sh[j] = st->s2; xb->top[j] = st->top; }
                    } else {
                        // lo_j = base of the coarse (key >> 20) bin that holds the k_j-th largest; XBINS bins of
                        // 2^10 keys cover that coarse bin, keys above it count as above the bracket
                        uint32_t b, ab, cn;
                        wave_locate_bin(p.coarse + (size_t)t * NBIN, 1, nullptr, seg_k(p, t, j), b, ab, cn);
                        if (b == NONE) { b = 0; if (lane == 0) p.status->error = 1; }
                        xb->lo[j] = b << 20;
                    }
                    if (xb->lo[j] != NONE) {
                        const uint64_t e = (uint64_t)xb->lo[j] + ((uint64_t)XBINS << xb->sh[j]);
                        xb->end[j] = e >= (uint64_t)KEY_END ? KEY_END : (uint32_t)e;
                        if (!narrow) xb->top[j] = xb->end[j];
                    }
                    xb->lo_min = xb->lo[j] < xb->lo_min ? xb->lo[j] : xb->lo_min;
                    if (j == p.commit) xb->lo_c = xb->lo[j];
                }
            }
        }
        c.lo_min = xb->lo_min; c.lo_c = c.split ? xb->lo_c : xb->lo_min;
        static_assert(EF || NCF == MAXCF, "the exact routes are compiled for any number of CFs");
#pragma unroll
        for (int j = 0; j < NCF; ++j) {
            if (j < p.n_cf) {
                c.lo[j] = xb->lo[j];
                c.sh[j] = xb->sh[j];
                c.top[j] = xb->end[j];
                if (first && c.lo[j] != NONE) {
                    // record the new bounds; clear what the refine pass may add to
                    CfState* st = &p.st[(size_t)t * p.n_cf + j];
                    if (lane == 0) {
                        st->lo = c.lo[j]; st->s = c.sh[j]; st->mode = MODE_FAIL; st->redo = 1;
                        if (!narrow) st->top = xb->end[j];
                    }
                    for (int i = lane; i < NBIN; i += 64) p.hist2[((size_t)t * p.n_cf + j) * NBIN + i] = 0;
                    if (lane < (int)seg_rep(p, t)) p.list_cnt[(seg_block(p, t, j) + lane) * 32] = 0;
                }
            }
        }
        // (on the narrow route the lists and the segment's candidate thresholds stay as they are)
        if (first && lane == 0 && !narrow) { p.seg[t].lo_min = c.lo_min; p.seg[t].lo_c = c.lo_c; p.seg[t].pz = NONE; }
    }
    // the copy of the histogram this wavefront adds to: spread by the sub-tile number, and by the tile number too,
    // because the narrow route's re-binning calls arrive with v = 8 u only
    c.hstride = seg_rep(p, t) * NBIN;
    c.h1 = p.hist1 + (seg_block(p, t, 0) + ((v ^ (v / SUB)) & (seg_rep(p, t) - 1u))) * NBIN;
    c.cidx = p.cand_idx + (size_t)v * TS;
    c.cval = p.cand_val + (size_t)v * TS;
    c.bkey = p.brk_key + (size_t)v * TS;
    c.bval = p.brk_val + (size_t)v * TS;
    c.run = 0;
    c.brun = 0;
    c.ssd = 0.0;

    if (narrow) {
        // the lists stay as they are; only the histograms of the CFs concerned are rebuilt, with the new bins, from
        // the tile's bracket lists.  Called for the first sub-tile of a tile only: the wavefront takes the whole tile.
        // An entry counts for CF j if it lies inside the bracket the lists were collected with (below top_j: what
        // lies above has been counted as above the bracket already) and from the located bin's first key on; past
        // that bin's last key it adds to the count above the new, narrower bracket.
        const TileRef tr = tile_ref(p, u);
        const uint32_t cnt = tr.tl.total();
        for (uint32_t i0 = 0; i0 < cnt; i0 += 64 * 8) {
            uint32_t kq[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t i = i0 + q * 64 + lane;
                float unused;
                kq[q] = 0;
                if (i < cnt) ref_entry(p, u, tr, i, kq[q], unused);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (i0 + q * 64 + lane >= cnt) continue;
#pragma unroll
                for (int j = 0; j < NCF; ++j) {
                    if (j < c.ncf && kq[q] >= c.lo[j] && kq[q] < xb->top[j]) {
                        if (kq[q] >= c.top[j]) c.ovn[j]++;
                        else atomicAdd(&c.h1[j * c.hstride + ((kq[q] - c.lo[j]) >> c.sh[j])], 1u);
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < NCF; ++j) {
            if (j < p.n_cf) {
                const uint32_t o = wave_sum(c.ovn[j]);
                if (lane == 0 && o) atomicAdd(&p.ovfc[(((size_t)t * p.n_cf + j) * 64 + (u & 63)) * 32], o);
            }
        }
        return;
    }

    bool dense = false;
    if (p.vec_ok && (s0 & 3) == 0 && e0 - s0 == TS) {
        // a whole sub-tile: the loads of all its rows first, then the arithmetic
        v4f x[ROWS], y[ROWS];
        v4i m[ROWS];
#pragma unroll
        for (int q = 0; q < ROWS; ++q) row_load<M>(p, s0 + q * ROW + 4 * lane, x[q], y[q], m[q]);
        float a[ROWS][4];
        uint32_t nc = 0;  // candidates for the message in this sub-tile
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            row_finish<M>(p, x[q], y[q], m[q], a[q]);
            uint32_t key[4];
            keys_of_row<RND, NCF>(c, a[q], s0 + q * ROW + 4 * lane, key);
#pragma unroll
            for (int e = 0; e < 4; ++e) nc += (uint32_t)__popcll(__ballot(key[e] >= c.lo_c));
        }
        dense = nc >= DENSE_SUB;
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const int64_t g = s0 + q * ROW + 4 * lane;
            uint32_t key[4];
            keys_of_row<RND, NCF>(c, a[q], g, key);
            if (M == SM_EF) {
                // acc goes back into the residual; in a sub-tile that keeps a candidate list an entry above the committed
                // CF's bracket leaves +0 there already: it is selected unless the bracket fails (the list keeps its value,
                // and the exact route puts it back), which spares the emit step a scattered store per selected entry
                v4f o;
                o.x = (!dense && key[0] >= c.pz) ? 0.0f : a[q][0];
                o.y = (!dense && key[1] >= c.pz) ? 0.0f : a[q][1];
                o.z = (!dense && key[2] >= c.pz) ? 0.0f : a[q][2];
                o.w = (!dense && key[3] >= c.pz) ? 0.0f : a[q][3];
                st_stream(o, (v4f*)(p.res + g));
            }
            consume<EF, RND, NCF>(c, a[q], key, g, 0xFu, !dense);
        }
    } else {
        // a ragged or unaligned sub-tile: element-wise, guarded; rows start at a multiple of 4 elements
        for (int64_t rb = s0 & ~(int64_t)3; rb < e0; rb += ROW) {
            const int64_t g = rb + 4 * lane;
            float a[4];
            unsigned vm = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t q = g + e;
                a[e] = 0.0f;
                if (q >= s0 && q < e0) {
                    vm |= 1u << e;
                    a[e] = element_load<M>(p, q);
                }
            }
            uint32_t key[4];
            keys_of_row<RND, NCF>(c, a, g, key);
            if (M == SM_EF) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((vm >> e) & 1u) p.res[g + e] = key[e] >= c.pz ? 0.0f : a[e];
            }
            consume<EF, RND, NCF>(c, a, key, g, vm, true);
        }
    }

#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        if (j < p.n_cf) {
            const uint32_t o = wave_sum(c.ovn[j]);
            const double s = wave_sum(c.ovs[j]);
            if (lane == 0) {
                p.ovn[(size_t)v * p.n_cf + j] = o;
                p.ovs[(size_t)v * p.n_cf + j] = s;
                if (o) atomicAdd(&p.ovfc[(((size_t)t * p.n_cf + j) * 64 + (v & 63)) * 32], o);
            }
        }
    }
    if (EF) {
        const double s = wave_sum(c.ssd);
        if (lane == 0) p.ssd[v] = s;
    }
    if (lane == 0) { p.cand_cnt[v] = dense ? DENSE_BIT : c.run; p.brk_cnt[v] = c.brun; }
}

// First pass (SM_EF, SM_SINGLE): one sub-tile per wavefront, one launch covers the whole gradient.
// SM_EXACT: a fixed number of wavefronts walks over all tiles (only those of failed segments do any work).
template <int M, bool RND, int NCF>
__global__ __launch_bounds__(WG) void stream_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t w = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + (threadIdx.x >> 6));
    if constexpr (M != SM_EXACT) {
        stream_subtile<M, RND, NCF>(p, w, lane, nullptr);
    } else {
        if (p.status->any_fail == 0) return;
        ExactBounds xb;
        xb.t = -1;
        const uint32_t nw = gridDim.x * WAVES;
        for (uint32_t u = w; u < p.n_tiles; u += nw) {
            const uint32_t kind = p.seg[tile_seg(p, u)].fail;
            if (kind == FAIL_NONE) continue;
            // FAIL_NARROW: one call re-bins the bracket lists of the whole tile; FAIL_FULL: sub-tile by sub-tile
            const int subs = (kind == FAIL_FULL) ? SUB : 1;
            for (int j = 0; j < subs; ++j) stream_subtile<SM_EXACT, RND, NCF>(p, u * SUB + j, lane, &xb);
        }
    }
}

// The candidates of sub-tile v that its first pass replaced by +0 in the residual get their values back (the
// sub-tile's candidate list holds them; nobody else touches the sub-tile).  By one wavefront.
__device__ __forceinline__ void put_back_subtile(const Params& p, uint32_t v, uint32_t pz, int lane)
{
    const uint32_t cc = p.cand_cnt[v];
    if (cc & DENSE_BIT) return;  // such a sub-tile kept acc
    const float* cv = p.cand_val + (size_t)v * TS;
    const int32_t* ci = p.cand_idx + (size_t)v * TS;
    for (uint32_t i0 = 0; i0 < cc; i0 += 64 * 4) {
        float vq[4];
        int32_t iq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t i = i0 + q * 64 + lane;
            vq[q] = cv[i < cc ? i : 0u];
            iq[q] = ci[i < cc ? i : 0u];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (i0 + q * 64 + lane < cc && cand_key(p, iq[q], vq[q]) >= pz) p.res[iq[q]] = vq[q];
    }
}

// ---------------------------------------------------------------------------------------------
// F1 (exact route, FAIL_FULL): histogram of key >> 20 over the tiles of failed segments; the wavefront
// of a failed segment's first tile also clears that segment's bracket histograms
// ---------------------------------------------------------------------------------------------
constexpr int CSUB = 8;  // copies of the coarse histogram inside a workgroup: lane l counts in copy l % CSUB

__global__ __launch_bounds__(WG) void coarse_kernel(Params p)
{
    // Gradient magnitudes crowd into a few exponents, so most lanes of a wavefront hit the same few bins and
    // LDS atomics on one copy serialise 64-fold; CSUB copies cut that to 64 / CSUB.
    // (a row is one word longer than the histogram, so that the CSUB counters of one bin lie in different banks)
    __shared__ uint32_t lh[CSUB][NBIN + 1];
    if (p.status->any_fail == 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t* h = lh[lane & (CSUB - 1)];
    // a fixed number of workgroups walks over the tiles (a workgroup takes WAVES consecutive tiles at a time, one per
    // wavefront), so that the launch costs little when nothing failed
    for (uint32_t i = tid; i < CSUB * (NBIN + 1); i += WG) (&lh[0][0])[i] = 0;
    __syncthreads();
    int cur = -1;  // segment whose counts sit in lh
    for (uint32_t u0 = blockIdx.x * WAVES; u0 < p.n_tiles; u0 += gridDim.x * WAVES) {
        // the workgroup's tiles may belong to different segments: one segment at a time, flushed in between
        const uint32_t u1 = u0 + WAVES < p.n_tiles ? u0 + WAVES : p.n_tiles;
        for (uint32_t ub = u0; ub < u1;) {
            const int t = tile_seg(p, ub);
            uint32_t ue = ub + 1;
            while (ue < u1 && tile_seg(p, ue) == t) ++ue;
            const uint32_t kind = p.seg[t].fail;
            if (kind == FAIL_FULL) {
                if (cur != t && cur >= 0) {
                    // flush the previous segment's counts
                    __syncthreads();
                    uint32_t* gh = p.coarse + (size_t)cur * NBIN;
                    for (uint32_t i = tid; i < NBIN; i += WG) {
                        uint32_t v = 0;
#pragma unroll
                        for (int c = 0; c < CSUB; ++c) { v += lh[c][i]; lh[c][i] = 0; }
                        if (v) atomicAdd(&gh[i], v);
                    }
                    __syncthreads();
                }
                cur = t;
                const uint32_t u = ub + (tid >> 6);
                if (u < ue) {
                    const int64_t sb = seg_begin(p, t), se = seg_end(p, t);
                    const int64_t s0 = sb + (int64_t)(u - seg_tile0(p, t)) * TW;
                    const int64_t e0 = (s0 + TW < se) ? s0 + TW : se;
                    if (u == seg_tile0(p, t)) {
                        for (uint32_t i = lane; i < (uint32_t)p.n_cf * seg_rep(p, t) * NBIN; i += 64) p.hist1[seg_block(p, t, 0) * NBIN + i] = 0;
                        for (int i = lane; i < p.n_cf * 64; i += 64) p.ovfc[((size_t)t * p.n_cf * 64 + i) * 32] = 0;
                    }
                    const uint32_t pz = p.single ? NONE : p.seg[t].pz;
                    if (pz != NONE) {
                        // acc is read again from the residual: first put back what the first pass replaced by +0 there
                        for (int j = 0; j < SUB; ++j) put_back_subtile(p, u * SUB + j, pz, lane);
                        __threadfence_block();  // the loads below are this wavefront's own, of the same addresses
                    }
                    for (int64_t q0 = s0 + lane; q0 < e0; q0 += 64 * 16) {
                        // all loads first, without branches around them (an element past the end reads the last
                        // one instead and is not counted), so that they are in flight together
                        float a[16];
#pragma unroll
                        for (int r = 0; r < 16; ++r) a[r] = p.acc[q0 + r * 64 < e0 ? q0 + r * 64 : e0 - 1];
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (q0 + r * 64 < e0) atomicAdd(&h[cand_key(p, (int32_t)(q0 + r * 64), a[r]) >> 20], 1u);
                    }
                }
            }
            ub = ue;
        }
    }
    if (cur >= 0) {
        __syncthreads();
        uint32_t* gh = p.coarse + (size_t)cur * NBIN;
        for (uint32_t i = tid; i < NBIN; i += WG) {
            uint32_t v = 0;
#pragma unroll
            for (int c = 0; c < CSUB; ++c) v += lh[c][i];
            if (v) atomicAdd(&gh[i], v);
        }
    }
}

// How the bin that holds the k-th largest gets resolved to one key.
struct BinPlan {
    uint32_t mode, base, span, above, c;
};

// Decide from the located bin (b, above, c) of the bracket histogram with bins (key - lo) >> s, of which the
// first nb are in use (anything from bin nb on was counted as above the bracket and arrives as bin OVF).
__device__ __forceinline__ BinPlan plan_bin(uint32_t lo, uint32_t s, uint32_t b, uint32_t above, uint32_t c)
{
    BinPlan q;
    if (b == NONE || b == OVF) q.mode = MODE_FAIL;  // fewer than k entries from lo on, or the k-th lies above the bracket
    else if (s == 0) q.mode = MODE_RESOLVED;
    else if (c <= LCAP) q.mode = MODE_GATHER;
    else if (s <= 11) q.mode = MODE_HIST;
    else q.mode = MODE_FAIL;
    q.base = (b == NONE || b == OVF) ? 0u : lo + (b << s);
    q.span = (1u << s) - 1u;
    q.above = above;
    q.c = c;
    return q;
}

__device__ __forceinline__ void store_plan(CfState* st, const BinPlan& q)
{
    st->mode = q.mode;
    if (q.mode != MODE_FAIL) {
        st->base = q.base; st->span = q.span; st->above = q.above; st->c = q.c;
        if (q.mode == MODE_RESOLVED) { st->tau = q.base; st->cnt_gt = q.above; st->need = st->k - q.above; }
    }
}

// ---------------------------------------------------------------------------------------------
// L1: one workgroup per (segment, CF): find the bracket-histogram bin of the k-th largest and
// decide how to resolve it; a segment whose bracket failed is marked for an exact route
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void locate_kernel(Params p)
{
    __shared__ uint32_t scratch[8];
    const int tid = threadIdx.x;
    const uint32_t id = blockIdx.x;
    const int t = id / p.n_cf, j = id - t * p.n_cf;
    if (seg_small(p, t)) return;
    CfState* st = &p.st[id];
    const uint32_t k = seg_k(p, t, j);
    const uint32_t lo = p.bnd_lo[id];
    uint32_t s, top;
    bracket_bins(lo, p.bnd_hi[id], s, top);
    uint32_t b, above, c;
    const uint32_t copies = seg_rep(p, t);
    team_locate_bin(p.hist1 + seg_block(p, t, j) * NBIN, (int)copies, p.ovfc + (size_t)id * 64 * 32, k, tid, scratch,
                    [] { __syncthreads(); }, b, above, c);
    const BinPlan q = plan_bin(lo, s, b, above, c);
    if (q.mode == MODE_HIST)
        for (int i = tid; i < NBIN; i += 256) p.hist2[(size_t)id * NBIN + i] = 0;
    const bool narrow = q.mode == MODE_FAIL && b != NONE && b != OVF;
    if (narrow) {
        // a bin 2^s keys wide (s > 11) with more than LCAP keys: XBINS bins of 2^(s - 10) keys cover it, and a
        // bin at most 2^10 keys wide can always be resolved (gathered or histogrammed key by key); this CF's
        // histogram is rebuilt by the exact route, the count above the bracket stays
        for (uint32_t i = tid; i < copies * NBIN; i += 256) p.hist1[seg_block(p, t, j) * NBIN + i] = 0;
    }
    if (tid == 0) {
        st->k = k; st->lo = lo; st->s = s; st->top = top;
        st->base = 0; st->span = 0; st->above = 0; st->c = 0; st->tau = 0; st->need = 0; st->cnt_gt = 0;
        st->redo = 0; st->lo2 = 0; st->s2 = 0; st->pad = 0;
        store_plan(st, q);
        if (q.mode == MODE_FAIL) {
            p.status->any_fail = 1;
            uint32_t kind = FAIL_FULL;
            if (narrow) {
                kind = FAIL_NARROW;
                st->redo = 1; st->lo2 = lo + (b << s); st->s2 = s - 10;
            }
            if (atomicMax(&p.seg[t].fail, kind) == 0u) atomicAdd(&p.status->n_fail, 1);
        }
        if (j == 0) {
            // what the segment's tiles need of all its CFs together
            uint32_t lo_min = NONE, lo_c = NONE, pz = NONE;
            for (int x = 0; x < p.n_cf; ++x) {
                const uint32_t lx = p.bnd_lo[(size_t)t * p.n_cf + x];
                lo_min = lx < lo_min ? lx : lo_min;
                if (x == p.commit) {
                    uint32_t sx, tx;
                    bracket_bins(lx, p.bnd_hi[(size_t)t * p.n_cf + x], sx, tx);
                    lo_c = lx;
                    pz = zero_from(p, t, lx, tx);
                }
            }
            p.seg[t].lo_min = lo_min; p.seg[t].lo_c = lo_c; p.seg[t].pz = pz;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// R1: one wavefront per tile.  The tile's sums of the pass over the gradient (energy, entries above
// every CF's bracket and their energy) are added up over its sub-tiles; then the tile's entries inside
// the brackets are walked: per CF, those above the bin that holds the k-th largest are counted and
// their energy summed, those inside that bin are gathered (key, tile, value) or histogrammed.  For a
// segment that took an exact route the plan is derived here, by every wavefront for itself, from the
// rebuilt bracket histogram (its first tile's wavefront records it).
// ---------------------------------------------------------------------------------------------
// (the form for four CFs is held to 80 registers, a dozen values spilled: six wavefronts per SIMD instead of four
// take the ResNet101 shape's tiles in one round instead of two)
// HEADS: the heads of the tile's lists are fetched before their lengths are known.  That pays where all tiles'
// wavefronts are resident at once and the kernel's time is one wavefront's chain of round trips to memory (the
// ResNet101 shape: 10.1 -> 7.9 us); with more tiles than that the chip is busy either way, and the extra loads and
// registers cost (the VGG16 shape: 10 -> 14 us), so the host picks the form by the number of tiles.
template <int NCF, bool HEADS>  // compiled for calls with up to NCF CFs: the loops over the CFs are unrolled
__global__ __launch_bounds__(LWG) __attribute__((amdgpu_waves_per_eu((NCF == 3 || NCF == 4) ? 6 : 1, 8))) void refine_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t u = __builtin_amdgcn_readfirstlane(blockIdx.x * LWAVES + (threadIdx.x >> 6));
    if (u >= p.n_tiles) return;
    // loads that depend on nothing but the tile number come first, so that they are in flight together
    const int any_fail = p.status->any_fail;
    const double ssd = lane < SUB ? p.ssd[(size_t)u * SUB + lane] : 0.0;
    // ... among them the heads of the tile's eight lists, before their lengths are known: lane l takes entries
    // l % 8 + 8 r (r < SPEC_R) of sub-tile l / 8.  A tile whose lists are no longer than that (most tiles of a call
    // with a CF of 100 or more) is done with one round trip to memory less.  Top-k keys only.
    constexpr int SPEC_R = HEADS ? 4 : 1;
    uint32_t spec[SPEC_R];
    if constexpr (HEADS) {
        const uint32_t* src = (p.split ? p.brk_key : (const uint32_t*)p.cand_val) + (size_t)u * TW + (size_t)(lane >> 3) * TS + (lane & 7);
#pragma unroll
        for (int r = 0; r < SPEC_R; ++r) spec[r] = src[8 * r];
    }
    uint32_t on[NCF];
    double os[NCF];
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        const bool have = lane < SUB && j < p.n_cf;
        on[j] = have ? p.ovn[((size_t)u * SUB + lane) * p.n_cf + j] : 0u;
        os[j] = have ? p.ovs[((size_t)u * SUB + lane) * p.n_cf + j] : 0.0;
    }
    const int t = tile_seg(p, u);
    // (the plan as the locate step left it: fetched with the counts, not after them)
    uint32_t mode[NCF], base[NCF], span[NCF], top[NCF];
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        mode[j] = MODE_RESOLVED; base[j] = NONE; span[j] = 0; top[j] = 0;
        if (j < p.n_cf) {
            const CfState* st = &p.st[(size_t)t * p.n_cf + j];
            mode[j] = st->mode; base[j] = st->base; span[j] = st->span; top[j] = st->top;
        }
    }
    const TileRef tr = tile_ref(p, u);
    const uint32_t cnt = tr.tl.total();
    const bool redo = any_fail != 0 && p.seg[t].fail != 0;
    const bool first = redo && (u == seg_tile0(p, t));
    uint32_t hn[NCF], tin = 0;
    double hs[NCF];
#pragma unroll
    for (int j = 0; j < NCF; ++j) { hn[j] = 0; hs[j] = 0.0; }
    if (cnt != 0 || first) {
        // exact route: the plan comes from the rebuilt bracket histogram.  A plain loop whose results go through
        // LDS, so that the search does not inflate the register count of the common path.
        __shared__ uint32_t rp[LWAVES][MAXCF][3];
        const int wib = threadIdx.x >> 6;
        if (redo) {
            const uint32_t fail_kind = p.seg[t].fail;
            if (first && lane == 0 && fail_kind == FAIL_NARROW) atomicAdd(&p.status->n_narrow, 1);
            for (int j = 0; j < p.n_cf; ++j) {
                CfState* st = &p.st[(size_t)t * p.n_cf + j];
                if (fail_kind == FAIL_NARROW && st->redo == 0) {
                    // this CF was not binned again: its plan stands (nobody writes it during this kernel)
                    if (lane == 0) { rp[wib][j][0] = st->mode; rp[wib][j][1] = st->base; rp[wib][j][2] = st->span; }
                    continue;
                }
                uint32_t b, above, c;
                wave_locate_bin(p.hist1 + seg_block(p, t, j) * NBIN, (int)seg_rep(p, t), p.ovfc + ((size_t)t * p.n_cf + j) * 64 * 32,
                                st->k, b, above, c);
                const BinPlan q = plan_bin(st->lo, st->s, b, above, c);
                if (lane == 0) {
                    rp[wib][j][0] = q.mode; rp[wib][j][1] = q.base; rp[wib][j][2] = q.span;
                    if (first) {
                        store_plan(st, q);
                        if (q.mode == MODE_FAIL) p.status->error = 1;  // the exact routes cannot fail
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // rp is read back by the same wavefront
        }
#pragma unroll
        for (int j = 0; j < NCF; ++j) {
            if (j < p.n_cf) {
                if (redo) {  // (an exact route may have moved the bracket's end too)
                    mode[j] = rp[wib][j][0]; base[j] = rp[wib][j][1]; span[j] = rp[wib][j][2];
                    top[j] = p.st[(size_t)t * p.n_cf + j].top;
                }
                if (mode[j] == MODE_FAIL) { base[j] = NONE; top[j] = 0; }  // (an error: nothing is counted)
            }
        }
        // what one entry adds, per CF whose bracket it lies in (below top_j: what lies above was counted by the pass)
        const auto take = [&](uint32_t key, float val, bool live) {
            const double dv = p.random ? (double)val : (double)__uint_as_float(key);  // Top-k: the key is |acc|
#pragma unroll
            for (int j = 0; j < NCF; ++j) {
                if (j >= p.n_cf) continue;
                const bool mine = live && key < top[j] && key >= base[j];
                if (__ballot(mine) == 0ull) continue;  // (most rounds hold nothing for the CFs with few entries)
                const bool in = mine && key - base[j] <= span[j];
                // Random-k: the entry at the threshold is the last one selected and has no particular magnitude, so a
                // bin that is one key wide adds its energy here (Top-k adds need * tau^2 in the scan instead)
                if (mine && (!in || (p.random && mode[j] == MODE_RESOLVED))) { hs[j] += dv * dv; hn[j] += in ? 0u : 1u; }
                if (j == p.commit && in) ++tin;
                if (mode[j] == MODE_GATHER) {
                    // one counter update per wavefront: the lanes with a key in the bin take consecutive slots
                    const uint64_t m = __ballot(in);
                    if (m != 0ull) {
                        const size_t lst = seg_block(p, t, j) + (blockIdx.x & (seg_rep(p, t) - 1u));
                        const int leader = __ffsll((unsigned long long)m) - 1;
                        uint32_t at = 0;
                        if (lane == leader) at = atomicAdd(&p.list_cnt[lst * 32], (uint32_t)__popcll(m));
                        at = __shfl(at, leader, 64);
                        const uint32_t pos = at + lanes_below(m);
                        if (in && pos < LCAP) {
                            p.list_key[lst * LCAP + pos] = key;
                            p.list_tile[lst * LCAP + pos] = u;
                            if (p.random) p.list_val[lst * LCAP + pos] = val;
                        }
                    }
                } else if (mode[j] == MODE_HIST && in) {
                    atomicAdd(&p.hist2[((size_t)t * p.n_cf + j) * NBIN + (key - base[j])], 1u);
                }
            }
        };
        // 64 entries per load and lane-row; eight loads in flight per lane where there are that many entries left, two
        // otherwise (most tiles hold a hundred entries or so, and a round that no lane has an entry for costs as many
        // instructions as a full one)
        uint32_t i0 = 0;
        if constexpr (HEADS) {
            // the lists' heads cover the tile if every list is its sub-tile's expected one and short enough
            bool heads = !p.random;
            const uint32_t expect = p.split ? 0u : 0xFFu;
#pragma unroll
            for (int j = 0; j < SUB; ++j) heads = heads && tr.tl.start[j + 1] - tr.tl.start[j] <= 8u * SPEC_R;
            if (heads && tr.main_mask == expect) {
                uint32_t mine_cnt = 0;
#pragma unroll
                for (int j = 0; j < SUB; ++j) if ((lane >> 3) == j) mine_cnt = tr.tl.start[j + 1] - tr.tl.start[j];
#pragma unroll
                for (int r = 0; r < SPEC_R; ++r) {
                    if (__ballot((uint32_t)(lane & 7) + 8u * r < mine_cnt) == 0ull) break;
                    take(spec[r] & 0x7FFFFFFFu, 0.0f, (uint32_t)(lane & 7) + 8u * r < mine_cnt);
                }
                i0 = cnt;
            }
        }
        if (i0 < cnt && cnt >= LONG_WALK && !p.random) {
            // long lists (a low CF, Top-k keys): sub-tile by sub-tile, so that no lane has to search for its entry's
            // slot.  A step's work is a fraction of a round trip to memory, and every wavefront of the launch is in
            // the same place, so the first two rounds of the next AHEAD sub-tiles are on their way while one is
            // worked on, whatever they hold; the words are carried as loaded and decoded where they are used
            // (decoded at once, the loads would be waited for at once).  The counts are the ones fetched with the
            // tile's first loads.
            constexpr int AHEAD = 4;
            const auto counts = [&](int j, uint32_t& c, bool& from_main) {
                c = 0;
#pragma unroll
                for (int x = 0; x < SUB; ++x) c = (x == j) ? tr.tl.start[x + 1] - tr.tl.start[x] : c;
                from_main = (tr.main_mask >> j) & 1u;
            };
            const auto fetch = [&](int j, uint32_t (&w)[2]) {
                const uint32_t* src = (((tr.main_mask >> j) & 1u) ? (const uint32_t*)p.cand_val : p.brk_key) + (size_t)u * TW + (size_t)j * TS;
#pragma unroll
                for (int q = 0; q < 2; ++q) w[q] = src[q * 64 + lane];
            };
            uint32_t wq[AHEAD][2];
#pragma unroll
            for (int a = 0; a < AHEAD; ++a) fetch(a, wq[a]);
            for (int j = 0; j < SUB; ++j) {
                uint32_t w0[2], c;
                bool fm;
#pragma unroll
                for (int q = 0; q < 2; ++q) w0[q] = wq[0][q];
#pragma unroll
                for (int a = 0; a + 1 < AHEAD; ++a) { wq[a][0] = wq[a + 1][0]; wq[a][1] = wq[a + 1][1]; }
                if (j + AHEAD < SUB) fetch(j + AHEAD, wq[AHEAD - 1]);
                counts(j, c, fm);
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if ((uint32_t)q * 64 < c) take(w0[q] & 0x7FFFFFFFu, 0.0f, q * 64 + lane < c);
                for (uint32_t b0 = 128; b0 < c; b0 += 128) {   // (a sub-tile with more than 128 such entries: rare)
                    const uint32_t* src = (fm ? (const uint32_t*)p.cand_val : p.brk_key) + (size_t)u * TW + (size_t)j * TS;
                    uint32_t kq[2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) kq[q] = src[(b0 + q * 64 + lane) & (TS - 1)] & 0x7FFFFFFFu;
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        if (b0 + q * 64 < c) take(kq[q], 0.0f, b0 + q * 64 + lane < c);
                }
            }
            i0 = cnt;
        }
        for (; i0 + 64 * 2 < cnt; i0 += 64 * 8) {
            uint32_t kq[8];
            float vq[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t i = i0 + q * 64 + lane;
                ref_entry(p, u, tr, i < cnt ? i : 0u, kq[q], vq[q]);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) take(kq[q], vq[q], i0 + q * 64 + lane < cnt);
        }
        if (i0 < cnt) {
            uint32_t kq[2];
            float vq[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const uint32_t i = i0 + q * 64 + lane;
                ref_entry(p, u, tr, i < cnt ? i : 0u, kq[q], vq[q]);
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) take(kq[q], vq[q], i0 + q * 64 + lane < cnt);
        }
    }
    // the tile's sums: what the pass over the gradient counted above the brackets, plus the above
    {
        const double x = wave_sum(ssd);
        if (lane == 0) p.ssd_t[u] = x;
    }
    tin = wave_sum(tin);
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        if (j < p.n_cf) {
            const uint32_t n = wave_sum(hn[j] + on[j]);
            // (the counted energy first, in sub-tile order, then the listed entries': a fixed order)
            const double e = wave_sum(os[j]) + wave_sum(hs[j]);
            if (lane == 0) {
                p.sss[(size_t)u * p.n_cf + j] = e;
                if (j == p.commit) { p.tg0[u] = n; p.tin[u] = tin; }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// SCAN: grid (n_seg, slices + n_cf), SCAN_T threads.  Every block first resolves one CF of its segment to
//       the exact key tau of the k-th largest (from the gathered keys by a bitwise search, or from the
//       key-by-key histogram), and how many keys equal to tau are selected.
//       Block (t, y < slices), committed CF: the counts of the y-th slice of SCAN_SLICE tiles of
//       segment t (entries above the located bin, plus the gathered entries above tau, by tile) and their
//       exclusive scan -> every tile's output offset and tie quota.  The totals of the earlier slices are
//       re-added by every block (a few batched loads), so no block waits on another.
//       Block (t, slices + j): statistics of (segment t, CF j), summed over the tiles in a fixed order.
// ---------------------------------------------------------------------------------------------
constexpr int SCAN_T = 1024;                 // threads
constexpr int SCAN_W = SCAN_T / 64;
constexpr int SCAN_PER = 4;                  // tiles per thread
constexpr int SCAN_SLICE = SCAN_T * SCAN_PER;
constexpr int LPER = LCAP / SCAN_T;          // gathered entries per thread
constexpr int RW = LPER;
constexpr int SPEC = SCAN_T / REP;           // threads that fetch the head of one gather list before its length is known
static_assert(LCAP % SCAN_T == 0 && SCAN_T % REP == 0 && SPEC * LPER <= LCAP && 2 * SCAN_T == NBIN,
              "the gathered entries are dealt evenly; a thread owns two bins of the search's histogram");

__global__ __launch_bounds__(SCAN_T) void scan_kernel(Params p, uint32_t slices)
{
    __shared__ uint32_t sg[SCAN_SLICE], se[SCAN_SLICE];
    __shared__ uint32_t wt[4][SCAN_W];
    __shared__ uint32_t wsum[2][SCAN_W];
    __shared__ double dred[3][SCAN_W];
    __shared__ uint64_t ured[SCAN_W];
    __shared__ uint32_t res3[3];
    const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    const int t = blockIdx.x;
    const bool scan_role = blockIdx.y < slices;
    const int j = scan_role ? p.commit : (int)(blockIdx.y - slices);
    const uint32_t id = (uint32_t)t * p.n_cf + j;
    const uint32_t u0 = seg_tile0(p, t), u1 = seg_tile1(p, t);
    const uint32_t slice0 = scan_role ? u0 + blockIdx.y * SCAN_SLICE : 0u;
    if ((scan_role && slice0 >= u1) || seg_small(p, t)) return;
    CfState* st = &p.st[id];

    // ---- loads that do not depend on the threshold come first, so that they overlap with its resolution
    // the fill counts of the gather lists and the plan
    const uint32_t copies = seg_rep(p, t);
    const size_t block0 = seg_block(p, t, j);
    uint32_t fill[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) fill[r] = (uint32_t)r < copies ? p.list_cnt[(block0 + r) * 32] : 0u;
    const uint32_t mode = st->mode, k = st->k, above = st->above, base = st->base, span = st->span, c = st->c;
    uint32_t tau = st->tau, need = st->need, cnt_gt = st->cnt_gt;   // valid if the located bin was one key wide
    // ... and the head of every gather list, SPEC * LPER entries of it, before the fill counts are known: a list is
    // rarely longer than that (the located bin's entries spread over the copies), and a load that waits for the
    // counts would cost this kernel another round trip to memory
    const uint32_t spec_r = (uint32_t)tid / SPEC;
    uint32_t sk[LPER], stl[LPER];
    float sv[LPER];
#pragma unroll
    for (int q = 0; q < LPER; ++q) {
        const size_t at = (block0 + (spec_r < copies ? spec_r : 0u)) * LCAP + (uint32_t)(tid % SPEC) + (uint32_t)q * SPEC;
        sk[q] = p.list_key[at];
        stl[q] = p.list_tile[at];
        sv[q] = p.random ? p.list_val[at] : 0.0f;
    }
    // scan: this slice, coalesced (entries above the located bin, entries inside it), and the totals of the
    // earlier slices of this segment; statistics: the tiles' sums, sixteen tiles per thread and round, fixed order
    uint32_t og[SCAN_PER], oi[SCAN_PER], pg = 0, pi = 0;
    double sd = 0.0, sj = 0.0;
    if (scan_role) {
#pragma unroll
        for (int q = 0; q < SCAN_PER; ++q) {
            const uint32_t u = slice0 + q * SCAN_T + tid;
            og[q] = (u < u1) ? p.tg0[u] : 0u;
            oi[q] = (u < u1) ? p.tin[u] : 0u;
        }
        for (uint32_t v0 = u0 + tid; v0 < slice0; v0 += 32 * SCAN_T) {
            uint32_t xg[32], xe[32];
#pragma unroll
            for (int q = 0; q < 32; ++q) {
                const uint32_t v = v0 + q * SCAN_T;
                xg[q] = (v < slice0) ? p.tg0[v] : 0u;
                xe[q] = (v < slice0) ? p.tin[v] : 0u;
            }
#pragma unroll
            for (int q = 0; q < 32; ++q) { pg += xg[q]; pi += xe[q]; }
        }
    } else {
        for (uint32_t v0 = u0 + tid; v0 < u1; v0 += 16 * SCAN_T) {
            double xd[16], xj[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const uint32_t u = v0 + q * SCAN_T;
                xd[q] = (u < u1) ? p.ssd_t[u] : 0.0;
                xj[q] = (u < u1) ? p.sss[(size_t)u * p.n_cf + j] : 0.0;
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) { sd += xd[q]; sj += xj[q]; }
        }
    }

    // ---- resolve (segment t, CF j)
    // This thread's gathered entries: key - base, tile, value, and which of the slots hold one (LPER per thread).
    uint32_t d[RW], rt[RW], live = 0;
    float rv[RW];
#pragma unroll
    for (int q = 0; q < RW; ++q) { d[q] = 0; rt[q] = 0; rv[q] = 0.0f; }
    if (mode == MODE_FAIL) {
        if (tid == 0) p.status->error = 1;
        tau = 0; need = 0; cnt_gt = 0;
    } else if (mode == MODE_HIST) {
        if (wib == 0) {
            uint32_t b, ab, cn;  // bins are single keys: base + b
            wave_locate_bin(p.hist2 + (size_t)id * NBIN, 1, nullptr, k - above, b, ab, cn);
            if (lane == 0) {
                if (b == NONE) { p.status->error = 1; b = 0; }
                res3[0] = base + b; res3[1] = above + ab;
            }
        }
        __syncthreads();
        tau = res3[0]; cnt_gt = res3[1]; need = k - cnt_gt;
    } else if (mode == MODE_GATHER) {
        // the want-th largest of the listed keys d = key - base.
        // The keys sit in REP lists; list r holds positions [off_r, off_r + n_r) of the concatenation.
        const uint32_t want = k - above;
        uint32_t off[REP + 1];
        off[0] = 0;
#pragma unroll
        for (int r = 0; r < REP; ++r) off[r + 1] = off[r] + fill[r];
        if (off[REP] != c || c > LCAP || want == 0 || want > c) {
            if (tid == 0) p.status->error = 1;
            tau = base; need = 0; cnt_gt = above;
        } else {
            bool spec_ok = true;
#pragma unroll
            for (int r = 0; r < REP; ++r) spec_ok = spec_ok && fill[r] <= (uint32_t)(SPEC * LPER);
            if (spec_ok) {
                // the entries are the ones fetched ahead: list spec_r, slots tid % SPEC + q SPEC
                uint32_t my_fill = 0;
#pragma unroll
                for (int r = 0; r < REP; ++r) if ((uint32_t)r == spec_r) my_fill = fill[r];   // (0 beyond the segment's copies)
#pragma unroll
                for (int q = 0; q < LPER; ++q) {
                    const uint32_t slot = (uint32_t)(tid % SPEC) + (uint32_t)q * SPEC;
                    d[q] = sk[q]; rt[q] = stl[q]; rv[q] = sv[q];
                    if (slot < my_fill) live |= 1u << q;
                }
            } else {
                // a long list: the entries are dealt over the block by their position in the concatenation; all loads
                // first, without branches around them (a position past the last key reads key 0 of the lists instead;
                // c >= 1 here), so that they are in flight together
#pragma unroll
                for (int q = 0; q < LPER; ++q) {
                    const uint32_t pos = (uint32_t)(q * SCAN_T + tid);
                    const uint32_t i = pos < c ? pos : 0u;
                    int r = 0;
#pragma unroll
                    for (int x = 1; x < REP; ++x) r += (i >= off[x]);
                    uint32_t o = 0;
#pragma unroll
                    for (int x = 0; x < REP; ++x) if (x == r) o = off[x];
                    const size_t at = (block0 + r) * LCAP + (i - o);
                    d[q] = p.list_key[at];
                    rt[q] = p.list_tile[at];
                    rv[q] = p.random ? p.list_val[at] : 0.0f;
                    if (pos < c) live |= 1u << q;
                }
            }
#pragma unroll
            for (int q = 0; q < LPER; ++q) d[q] = ((live >> q) & 1u) ? d[q] - base : 0u;
            // The want-th largest d: a histogram of 11 bits of d at a time, from the top bits down (one round unless
            // the located bin is more than 2048 keys wide), among the entries that agree with the bits found so far.
            // Thread tid owns bins 2047 - 2 tid and 2046 - 2 tid, so that a scan over the threads runs from the top bin.
            int nbits = 0;
            while (nbits < 32 && (span >> nbits) != 0u) ++nbits;
            uint32_t prefix = 0, pmask = 0, gsum = 0, left = want;
            int shift = nbits > 11 ? nbits - 11 : 0;
            for (;;) {
                sg[2 * tid] = 0; sg[2 * tid + 1] = 0;
                __syncthreads();
#pragma unroll
                for (int q = 0; q < LPER; ++q)
                    if (((live >> q) & 1u) && (d[q] & pmask) == prefix) atomicAdd(&sg[(d[q] >> shift) & (NBIN - 1)], 1u);
                __syncthreads();
                const uint32_t bA = (uint32_t)(NBIN - 1 - 2 * tid), bB = bA - 1u;
                const uint32_t hA = sg[bA], hB = sg[bB], mine = hA + hB;
                const uint32_t incl = wave_scan(mine);
                if (lane == 63) wsum[0][wib] = incl;
                __syncthreads();
                uint32_t higher = incl - mine;   // entries in the bins above this thread's two
#pragma unroll
                for (int w = 0; w < SCAN_W; ++w) if (w < wib) higher += wsum[0][w];
                if (higher < left && higher + hA >= left) { res3[0] = bA; res3[1] = higher; }
                else if (higher + hA < left && higher + mine >= left) { res3[0] = bB; res3[1] = higher + hA; }
                __syncthreads();
                prefix |= res3[0] << shift;
                pmask |= (uint32_t)(NBIN - 1) << shift;
                gsum += res3[1];
                left -= res3[1];
                if (shift == 0) break;
                shift = shift > 11 ? shift - 11 : 0;
                __syncthreads();   // (res3 and the histogram are rewritten in the next round)
            }
            tau = base + prefix; cnt_gt = above + gsum; need = k - cnt_gt;
            __syncthreads();
        }
    }
    const uint32_t dtau = tau - base;  // the threshold inside the located bin

    if (scan_role) {
        // (the plan itself stays as it is: the segment's other blocks are reading it)
        if (blockIdx.y == 0 && tid == 0) { st->tau = tau; st->need = need; st->cnt_gt = cnt_gt; }
        // entries equal to tau: those inside a located bin that is one key wide
        uint32_t pe = (mode == MODE_RESOLVED) ? pi : 0u;
#pragma unroll
        for (int q = 0; q < SCAN_PER; ++q) {
            sg[q * SCAN_T + tid] = og[q];
            se[q * SCAN_T + tid] = (mode == MODE_RESOLVED) ? oi[q] : 0u;
        }
        __syncthreads();
        if (mode == MODE_GATHER) {
            // the gathered entries above and at the threshold, by tile
#pragma unroll
            for (int q = 0; q < RW; ++q) {
                if (!((live >> q) & 1u) || d[q] < dtau) continue;
                const bool gt = d[q] > dtau;
                if (rt[q] < slice0) { if (gt) ++pg; else ++pe; }
                else if (rt[q] - slice0 < (uint32_t)SCAN_SLICE) atomicAdd(gt ? &sg[rt[q] - slice0] : &se[rt[q] - slice0], 1u);
            }
        } else if (mode == MODE_HIST) {
            // more keys in the located bin than a gather list holds (a mass of equal values): the tiles that have
            // entries in the bin are walked again, up to the end of this slice, one wavefront per tile at a time
            const uint32_t uend = slice0 + SCAN_SLICE < u1 ? slice0 + SCAN_SLICE : u1;
            const uint32_t top = st->top;
            for (uint32_t u = u0 + wib; u < uend; u += SCAN_W) {
                if (p.tin[u] == 0) continue;
                const TileRef tr = tile_ref(p, u);
                const uint32_t cnt = tr.tl.total();
                uint32_t g = 0, e = 0;
                for (uint32_t i = lane; i < cnt; i += 64) {
                    uint32_t key;
                    float unused;
                    ref_entry(p, u, tr, i, key, unused);
                    if (key < top && key >= base && key - base <= span) { g += key > tau; e += key == tau; }
                }
                g = wave_sum(g); e = wave_sum(e);
                if (lane == 0) {
                    if (u < slice0) { pg += g; pe += e; }
                    else { atomicAdd(&sg[u - slice0], g); atomicAdd(&se[u - slice0], e); }
                }
            }
        }
        pg = wave_sum(pg);
        pe = wave_sum(pe);
        if (lane == 0) { wt[2][wib] = pg; wt[3][wib] = pe; }
        __syncthreads();
        // this thread's SCAN_PER consecutive tiles
        uint32_t g[SCAN_PER], e[SCAN_PER], sum_g = 0, sum_e = 0;
#pragma unroll
        for (int i = 0; i < SCAN_PER; ++i) {
            g[i] = sg[tid * SCAN_PER + i]; e[i] = se[tid * SCAN_PER + i];
            sum_g += g[i]; sum_e += e[i];
        }
        const uint32_t ig = wave_scan(sum_g), ie = wave_scan(sum_e);
        if (lane == 63) { wt[0][wib] = ig; wt[1][wib] = ie; }
        __syncthreads();
        uint32_t run_g = ig - sum_g, run_e = ie - sum_e;   // counts before this thread's tiles
#pragma unroll
        for (int w = 0; w < SCAN_W; ++w) {
            if (w < wib) { run_g += wt[0][w]; run_e += wt[1][w]; }
            run_g += wt[2][w];
            run_e += wt[3][w];
        }
        uint32_t off[SCAN_PER], tk[SCAN_PER];
#pragma unroll
        for (int i = 0; i < SCAN_PER; ++i) {
            const uint32_t ties_before = run_e < need ? run_e : need;  // ties selected in earlier tiles
            const uint32_t left = need - ties_before;
            off[i] = run_g + ties_before;                               // output offset of the tile
            tk[i] = left < e[i] ? left : e[i];                          // its tie quota
            run_g += g[i];
            run_e += e[i];
        }
        // the number of pairs a tile emits is written by the thread that holds its counts
#pragma unroll
        for (int i = 0; i < SCAN_PER; ++i) {
            const uint32_t u = slice0 + tid * SCAN_PER + i;
            if (u < u1) p.tsel[u] = g[i] + tk[i];
        }
        // threshold sparsifier: how many entries are kept is only known here (the last thread of the last slice has
        // counted them all); the emit step emits them if they fit the caller's buffers
        if (p.bounds_from == BOUNDS_FIXED && tid == SCAN_T - 1 && slice0 + SCAN_SLICE >= u1) {
            p.status->count = (int)run_g;
            if (p.out_count) *p.out_count = (int64_t)run_g;
        }
#pragma unroll
        for (int i = 0; i < SCAN_PER; ++i) {
            sg[tid * SCAN_PER + i] = off[i];
            se[tid * SCAN_PER + i] = tk[i];
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < SCAN_PER; ++q) {
            const uint32_t u = slice0 + q * SCAN_T + tid;
            if (u < u1) { p.toff[u] = sg[q * SCAN_T + tid]; p.ttake[u] = se[q * SCAN_T + tid]; }
        }
        return;
    }

    // ---- statistics of (segment t, CF j)
    // the entries of the located bin above the threshold (Random-k: and the one at it).  Their order in the gather
    // lists varies from run to run, so their energies are added as integers: every square, exact in binary64, is
    // scaled by a power of two that puts the largest of them below 2^50 and truncated, the sum of up to LCAP of them
    // fits 64 bits and does not depend on the order, and it is off by less than 2^-38 of itself.
    double ebin = 0.0;
    if (mode == MODE_GATHER) {
        const auto square = [&](int q) {
            const bool in = ((live >> q) & 1u) && (d[q] > dtau || (p.random && d[q] == dtau));
            const double dv = p.random ? (double)rv[q] : (double)__uint_as_float(base + d[q]);
            return in ? dv * dv : 0.0;
        };
        const uint32_t kmax = base + span;   // the located bin's largest key
        if (!p.random && kmax < 0x7F800000u) {
            // Top-k keys are magnitudes, and the bin's own bounds say how large a square can get: no look at the
            // entries for the scale, and nothing can be infinite or NaN
            if (kmax != 0u) {
                const double m = (double)__uint_as_float(kmax);
                const int ex = ilogb(m * m);                  // every square is below 2^(ex + 1)
                const double sc = scalbn(1.0, 49 - ex);       // (a power of two: the product is exact)
                uint64_t acc = 0;
#pragma unroll
                for (int q = 0; q < RW; ++q) acc += (uint64_t)(square(q) * sc);   // < 2^50 each
                acc = wave_sum(acc);
                if (lane == 0) ured[wib] = acc;
                __syncthreads();
                uint64_t all = 0;
#pragma unroll
                for (int w = 0; w < SCAN_W; ++w) all += ured[w];
                ebin = scalbn((double)all, ex - 49);
            }
        } else {
        double mx = 0.0, plain = 0.0;
        bool finite = true;
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const double x = square(q);
            mx = fmax(mx, x);   // (a NaN square is skipped here and shows in the plain sum)
            plain += x;
            finite = finite && (x <= 1.0e300);
        }
        mx = wave_max(mx);
        if (lane == 0) dred[2][wib] = mx;
        const bool all_finite = __syncthreads_and(finite ? 1 : 0) != 0;
        mx = 0.0;
#pragma unroll
        for (int w = 0; w < SCAN_W; ++w) mx = fmax(mx, dred[2][w]);
        __syncthreads();
        if (!all_finite) {
            // an infinite or NaN square: the sum is infinite or NaN in any order
            plain = wave_sum(plain);
            if (lane == 0) dred[2][wib] = plain;
            __syncthreads();
            for (int w = 0; w < SCAN_W; ++w) ebin += dred[2][w];
        } else if (mx > 0.0) {
            const int ex = ilogb(mx);                      // 2^ex <= mx < 2^(ex + 1)
            uint64_t acc = 0;
#pragma unroll
            for (int q = 0; q < RW; ++q) acc += (uint64_t)scalbn(square(q), 49 - ex);   // < 2^50 each
            acc = wave_sum(acc);
            if (lane == 0) ured[wib] = acc;
            __syncthreads();
            uint64_t all = 0;
#pragma unroll
            for (int w = 0; w < SCAN_W; ++w) all += ured[w];
            ebin = scalbn((double)all, ex - 49);
        }
        }
    } else if (mode == MODE_HIST) {
        // Top-k only (priorities are distinct): the key-by-key histogram's bins above the threshold, in bin order
        double s = 0.0;
        for (uint32_t b = tid; b < NBIN; b += SCAN_T) {
            const uint32_t cn = (b > dtau && b <= span) ? p.hist2[(size_t)id * NBIN + b] : 0u;
            const double dv = (double)__uint_as_float(base + b);
            s += (double)cn * (dv * dv);
        }
        s = wave_sum(s);
        if (lane == 0) dred[2][wib] = s;
        __syncthreads();
        for (int w = 0; w < SCAN_W; ++w) ebin += dred[2][w];
    }
    // every wavefront's sum, then the SCAN_W of them in order: the same order in every run
    {
        const double wd = wave_sum(sd), wj = wave_sum(sj);
        if (lane == 0) { dred[0][wib] = wd; dred[1][wib] = wj; }
    }
    __syncthreads();
    if (tid == 0) {
        // fourth statistic: the threshold as a magnitude (Top-k) or as a priority (Random-k)
        const double tauv = p.random ? (double)tau : (double)__uint_as_float(tau);
        double ss_dense = 0.0, ss_above = 0.0;
        for (int w = 0; w < SCAN_W; ++w) { ss_dense += dred[0][w]; ss_above += dred[1][w]; }
        // Top-k: the ties all have magnitude tau; Random-k: the entry at the threshold has been summed
        const double ss_sel = ss_above + ebin + (p.random ? 0.0 : (double)need * tauv * tauv);
        double* o = p.out_stats + (size_t)id * GRAVAC_STATS_PER_CF;
        o[0] = ss_sel;
        o[1] = ss_dense;
        o[2] = (ss_dense == 0.0) ? 1.0 : ss_sel / ss_dense;
        o[3] = p.bounds_from == BOUNDS_FIXED ? (double)__uint_as_float(p.fixed_key) : tauv;
        if (j != p.commit) { st->tau = tau; st->need = need; st->cnt_gt = cnt_gt; }
    }
}

// ---------------------------------------------------------------------------------------------
// K4: one wavefront per tile emits the tile's share of the committed selection in ascending index
//     order and zeroes its residual slots.  A sub-tile with a candidate list is emitted from the list;
//     a sub-tile without one (mostly candidates) is read again, 1024 elements, and its residual rewritten.
// ---------------------------------------------------------------------------------------------
struct EmitCtx {
    uint32_t tau, take, pz;
    bool put_back;
    bool zero;   // selected entries are removed from the residual (not in a call without commit)
    int64_t pos, lim;
    uint32_t erun;
};

// One round of up to 64 listed candidates (idx, val), one per lane.
template <bool GEN>
__device__ __forceinline__ void emit_listed(const Params& p, EmitCtx& x, int32_t idx, float val, bool live)
{
    const bool rnd = GEN && p.random, single = GEN && p.single;
    const uint32_t key = rnd ? priority_of(p.rk_s0, p.rk_s1, (uint32_t)idx) : key_of(val);
    const bool gt = live && key > x.tau, eq = live && key == x.tau;
    const uint64_t me = __ballot(eq);
    bool sel = gt;
    if (me != 0ull) sel = gt || (eq && (x.erun + lanes_below(me)) < x.take);  // (few rounds hold a tie)
    const uint64_t ms = __ballot(sel);
    // the wavefront's pairs go to consecutive places from pos on: a uniform base and a small offset per lane
    const int64_t left = x.lim - x.pos;
    const uint32_t room = left >= 64 ? 64u : (left > 0 ? (uint32_t)left : 0u);
    float* ov = p.out_val + x.pos;
    int32_t* oi = p.out_idx + x.pos;
    if (sel) {
        const uint32_t o = lanes_below(ms);
        if (o < room) {
            ov[o] = val;
            if (!single) {
                oi[o] = idx;
                if (x.zero && key < x.pz) p.res[idx] = 0.0f;
            } else {
                const int mi = p.map_idx[idx];  // position in the message -> index in the gradient
                oi[o] = mi;
                if (p.restore && (uint64_t)(int64_t)mi < (uint64_t)p.n_restore) p.restore[mi] = 0.0f;
            }
        } else {
            p.status->error = 1;  // cannot happen if the counts are consistent; never write out of range
        }
    } else if (x.put_back && live && key >= x.pz) {
        p.res[idx] = val;
    }
    x.pos += __popcll(ms);
    x.erun += (uint32_t)__popcll(me);
}

// GEN false: compiled for the plain call (Top-k or threshold keys, gradient + residual).
// HEADS (plain call only): the heads of the tile's eight lists, 32 candidates each, are fetched with the kernel's first
// loads, before the lists' lengths are known; a tile whose lists are no longer than that is emitted from them, a
// lane's four consecutive candidates at a time, one round trip to memory earlier.  As in the refine kernel this
// pays where all tiles' wavefronts are resident at once, and the host picks the form by the number of tiles.
template <bool GEN, bool HEADS>
__global__ __launch_bounds__(LWG) __attribute__((amdgpu_waves_per_eu(HEADS ? 6 : 1, 8))) void emit_kernel(Params p)
{
    static_assert(!(GEN && HEADS), "the early loads exist in the plain form only");
    const bool rnd = GEN && p.random, single = GEN && p.single;  // (known to be off in the plain form)
    const int lane = threadIdx.x & 63;
    const uint32_t u = __builtin_amdgcn_readfirstlane(blockIdx.x * LWAVES + (threadIdx.x >> 6));
    if (u >= p.n_tiles) return;
    v4i hi4 = {0, 0, 0, 0};
    v4f hv4 = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (HEADS) {
        // lane l: candidates 4 (l % 8) .. + 3 of sub-tile l / 8 (16-byte aligned: a sub-tile's slots start at a multiple of TS)
        const size_t at = (size_t)u * TW + (size_t)(lane >> 3) * TS + 4u * (lane & 7);
        hi4 = *(const v4i*)(p.cand_idx + at);
        hv4 = *(const v4f*)(p.cand_val + at);
    }
    uint32_t cc[SUB];
    uint32_t dmask = 0;  // bit j: sub-tile j keeps no candidate list
#pragma unroll
    for (int j = 0; j < SUB; ++j) { cc[j] = p.cand_cnt[(size_t)u * SUB + j]; dmask |= (cc[j] & DENSE_BIT) ? 1u << j : 0u; }
    const bool any_dense = dmask != 0u;
    const int t = tile_seg(p, u);
    EmitCtx x;
    x.take = p.ttake[u];
    x.tau = p.st[(size_t)t * p.n_cf + p.commit].tau;
    // The first pass has left +0 in the residual of its listed sub-tiles for keys >= pz (not on the full exact route,
    // which has put acc back).  Those entries need no store here if they are selected, and get acc back if they are
    // not, which can only be when the threshold turned out to lie at or above pz.
    x.pz = (single || p.seg[t].fail == FAIL_FULL) ? NONE : p.seg[t].pz;
    x.put_back = x.pz != NONE && x.tau >= x.pz;
    x.zero = !p.no_commit;
    if (p.bounds_from == BOUNDS_FIXED && (int64_t)p.status->count > p.total_out) {
        // threshold sparsifier, more entries kept than the caller's buffers hold: nothing is emitted and nothing removed.
        // The listed sub-tiles get back the values the pass replaced by +0; the others kept acc.
        for (int j = 0; j < SUB; ++j) put_back_subtile(p, u * SUB + j, x.pz, lane);
        return;
    }
    if (p.tsel[u] == 0 && !x.put_back) return;
    const int64_t seg_out = seg_koff(p, t);
    x.lim = seg_out + (int64_t)seg_k(p, t, p.commit);  // end of this segment's message
    x.pos = seg_out + (int64_t)p.toff[u];
    x.erun = 0;
    const float* cv = p.cand_val + (size_t)u * TW;
    const int32_t* ci = p.cand_idx + (size_t)u * TW;
    if constexpr (HEADS) {
        bool covered = !any_dense;
        uint32_t cj = 0;  // candidates of this lane's sub-tile
#pragma unroll
        for (int j = 0; j < SUB; ++j) {
            covered = covered && cc[j] <= 32u;
            if ((lane >> 3) == j) cj = cc[j];
        }
        if (covered) {
            const int32_t ia[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
            const float va[4] = {hv4.x, hv4.y, hv4.z, hv4.w};
            uint32_t key[4];
            bool live[4], sel[4];
            uint32_t n_eq = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                live[e] = 4u * (lane & 7) + e < cj;
                key[e] = key_of(va[e]);
                sel[e] = live[e] && key[e] > x.tau;
                n_eq += (live[e] && key[e] == x.tau) ? 1u : 0u;
            }
            if (__ballot(n_eq != 0u) != 0ull) {
                // ties at the threshold: the first x.take of them in index order (lanes are in index order) are selected
                uint32_t rank = wave_scan(n_eq) - n_eq;   // ties in lower lanes
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (live[e] && key[e] == x.tau) { sel[e] = rank < x.take; ++rank; }
                }
            }
            const uint32_t n_sel = (sel[0] ? 1u : 0u) + (sel[1] ? 1u : 0u) + (sel[2] ? 1u : 0u) + (sel[3] ? 1u : 0u);
            uint32_t o = wave_scan(n_sel) - n_sel;       // pairs of lower lanes
            const int64_t left = x.lim - x.pos;
            const uint32_t room = left >= (int64_t)TW ? (uint32_t)TW : (left > 0 ? (uint32_t)left : 0u);
            float* ov = p.out_val + x.pos;
            int32_t* oi = p.out_idx + x.pos;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (sel[e]) {
                    if (o < room) {
                        ov[o] = va[e];
                        oi[o] = ia[e];
                        if (x.zero && key[e] < x.pz) p.res[ia[e]] = 0.0f;
                    } else {
                        p.status->error = 1;  // cannot happen if the counts are consistent; never write out of range
                    }
                    ++o;
                } else if (x.put_back && live[e] && key[e] >= x.pz) {
                    p.res[ia[e]] = va[e];
                }
            }
            return;
        }
    }
    TileLists tl;
    tl.start[0] = 0;
#pragma unroll
    for (int j = 0; j < SUB; ++j) tl.start[j + 1] = tl.start[j] + (cc[j] & ~DENSE_BIT);
    if (!any_dense && tl.total() < LONG_WALK) {
        // all sub-tiles listed, and shortly: their lists are walked as one, 64 candidates per round.  The loads of
        // the next rounds are issued before this round is worked on (an absent candidate reads slot 0 and is not
        // used), so that a wavefront does not wait a full round trip per round
        const uint32_t cnt = tl.total();
        float vn[4];
        int32_t in[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t q = r * 64 + lane;
            const uint32_t sl = (q < cnt) ? tl.slot(q) : 0u;
            vn[r] = cv[sl];
            in[r] = ci[sl];
        }
        for (uint32_t b0 = 0; b0 < cnt; b0 += 64 * 4) {
            float vq[4];
            int32_t iq[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) { vq[r] = vn[r]; iq[r] = in[r]; }
            if (b0 + 64 * 4 < cnt) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t q = b0 + 64 * 4 + r * 64 + lane;
                    const uint32_t sl = (q < cnt) ? tl.slot(q) : 0u;
                    vn[r] = cv[sl];
                    in[r] = ci[sl];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (b0 + r * 64 >= cnt) break;  // (a round that no lane has a candidate for costs as much as a full one)
                emit_listed<GEN>(p, x, iq[r], vq[r], b0 + r * 64 + lane < cnt);
            }
        }
        return;
    }
    if (!any_dense) {
        // all sub-tiles listed, at length (a low CF): sub-tile by sub-tile, so that no lane has to search for its
        // candidate's slot, and the first two rounds of every sub-tile are loaded before any is worked on: the
        // wavefront pays one round trip to memory, not one per sub-tile
        float va[SUB][2];
        int32_t ia[SUB][2];
#pragma unroll
        for (int j = 0; j < SUB; ++j) {
#pragma unroll
            for (int r = 0; r < 2; ++r) { va[j][r] = cv[j * TS + r * 64 + lane]; ia[j][r] = ci[j * TS + r * 64 + lane]; }
        }
#pragma unroll
        for (int j = 0; j < SUB; ++j) {
            const uint32_t c = cc[j];
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if ((uint32_t)r * 64 < c) emit_listed<GEN>(p, x, ia[j][r], va[j][r], r * 64 + lane < c);
            for (uint32_t b0 = 128; b0 < c; b0 += 128) {   // (more than 128 candidates and still listed)
                float vq[2];
                int32_t iq[2];
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const uint32_t q = (b0 + r * 64 + lane) & (TS - 1);
                    vq[r] = cv[j * TS + q];
                    iq[r] = ci[j * TS + q];
                }
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    if (b0 + r * 64 < c) emit_listed<GEN>(p, x, iq[r], vq[r], b0 + r * 64 + lane < c);
            }
        }
        return;
    }
    // sub-tile by sub-tile: a tile with sub-tiles that keep no list
    // (two rows of a sub-tile at a time: with room for a whole sub-tile the LDS of a workgroup would limit the
    // kernel to five wavefronts per SIMD, and the listed tiles of the same launch need the occupancy)
    __shared__ int32_t stage_idx[LWAVES][TS / 2];   // half a sub-tile's part of the message, per wavefront
    __shared__ float stage_val[LWAVES][TS / 2];
    int32_t* sidx = stage_idx[threadIdx.x >> 6];
    float* sval = stage_val[threadIdx.x >> 6];
    const int64_t tile0 = seg_begin(p, t) + (int64_t)(u - seg_tile0(p, t)) * TW;
    v4f nxt[ROWS];  // the rows of the next sub-tile without a list
    {
        const int64_t sn = tile0 + (int64_t)(__ffs((int)dmask) - 1) * TS;
#pragma unroll
        for (int q = 0; q < ROWS; ++q) nxt[q] = *(const v4f*)(p.acc + sn + q * ROW + 4 * lane);
    }
    // the first two rounds of the next sub-tile's list, loaded while this one is worked on, whatever they hold
    float vnx[2];
    int32_t inx[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) { vnx[r] = cv[r * 64 + lane]; inx[r] = ci[r * 64 + lane]; }
    for (int j = 0; j < SUB; ++j) {
        float vq[2];
        int32_t iq[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) { vq[r] = vnx[r]; iq[r] = inx[r]; }
        if (j + 1 < SUB) {
#pragma unroll
            for (int r = 0; r < 2; ++r) { vnx[r] = cv[(j + 1) * TS + r * 64 + lane]; inx[r] = ci[(j + 1) * TS + r * 64 + lane]; }
        }
        if (!((dmask >> j) & 1u)) {
            const uint32_t c = p.cand_cnt[(size_t)u * SUB + j];
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if ((uint32_t)r * 64 < c) emit_listed<GEN>(p, x, iq[r], vq[r], r * 64 + lane < c);
            for (uint32_t b0 = 128; b0 < c; b0 += 128) {   // (more than 128 candidates and still listed)
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const uint32_t q = (b0 + r * 64 + lane) & (TS - 1);
                    vq[r] = cv[j * TS + q];
                    iq[r] = ci[j * TS + q];
                }
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    if (b0 + r * 64 < c) emit_listed<GEN>(p, x, iq[r], vq[r], b0 + r * 64 + lane < c);
            }
            continue;
        }
        // a whole, aligned sub-tile that kept acc in the residual (or is the message itself, single-source mode):
        // four rows of 256 elements, a lane's four consecutive elements at a time.  Its rows were loaded while the
        // sub-tile before it was worked on; now the next such sub-tile's loads are issued.
        const int64_t s0 = tile0 + (int64_t)j * TS;
        uint32_t staged = 0;  // pairs in LDS so far
        v4f av[ROWS];
#pragma unroll
        for (int q = 0; q < ROWS; ++q) av[q] = nxt[q];
        {
            const uint32_t later = dmask & ~((2u << j) - 1u);
            if (later != 0u) {
                const int64_t sn = tile0 + (int64_t)(__ffs((int)later) - 1) * TS;
#pragma unroll
                for (int q = 0; q < ROWS; ++q) nxt[q] = *(const v4f*)(p.acc + sn + q * ROW + 4 * lane);
            }
        }
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const int64_t g = s0 + q * ROW + 4 * lane;
            const float a[4] = {av[q].x, av[q].y, av[q].z, av[q].w};
            bool gt[4], eq[4], sel[4];
            uint32_t ties_below = 0;   // ties in lower lanes of this row
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t key = rnd ? priority_of(p.rk_s0, p.rk_s1, (uint32_t)(g + e)) : key_of(a[e]);
                gt[e] = key > x.tau;
                eq[e] = key == x.tau;
            }
            uint32_t ties_row = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint64_t m = __ballot(eq[e]);
                ties_below += lanes_below(m);
                ties_row += (uint32_t)__popcll(m);
            }
            uint32_t er = x.erun + ties_below;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sel[e] = gt[e] || (eq[e] && er < x.take);
                er += eq[e] ? 1u : 0u;
            }
            uint32_t pre = 0, tot = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint64_t m = __ballot(sel[e]);
                pre += lanes_below(m);
                tot += (uint32_t)__popcll(m);
            }
            // the selected pairs go to their place in the sub-tile's part of the message, in LDS first
            uint32_t o = staged + pre;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (!sel[e]) continue;
                int32_t gi = (int32_t)(g + e);
                if (single) {
                    gi = p.map_idx[g + e];
                    if (p.restore && (uint64_t)(int64_t)gi < (uint64_t)p.n_restore) p.restore[gi] = 0.0f;
                }
                sidx[o] = gi;
                sval[o] = a[e];
                ++o;
            }
            if (!single && x.zero) {
                v4f r;
                r.x = sel[0] ? 0.0f : a[0]; r.y = sel[1] ? 0.0f : a[1];
                r.z = sel[2] ? 0.0f : a[2]; r.w = sel[3] ? 0.0f : a[3];
                *(v4f*)(p.res + g) = r;
            }
            staged += tot;
            x.erun += ties_row;
            if (q & 1) {
                // ... and from there into the message, 64 consecutive pairs per store
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // the wavefront's own LDS writes, read back by other lanes
                if (x.pos + (int64_t)staged > x.lim) p.status->error = 1;  // cannot happen if the counts are consistent
                for (uint32_t i = lane; i < staged; i += 64) {
                    if (x.pos + i < x.lim) {   // never write out of range
                        p.out_idx[x.pos + i] = sidx[i];
                        p.out_val[x.pos + i] = sval[i];
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // read before the next rows overwrite them
                x.pos += staged;
                staged = 0;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// decompression: dense_out[idx] += val, workers in order.  A workgroup owns one tile of DTILE floats
// of dense_out at a time (tiles are dealt round-robin over a fixed number of workgroups).  A tile
// that lies outside every message's index range is skipped without touching memory.  Otherwise the
// tile's range in every worker's index-sorted message is found by a 32-way search (32 threads per
// worker, both ends at once, 8 workers at a time); if any message touches the tile it is loaded
// into LDS, the pairs are applied worker by worker (indices within one worker are unique, so plain
// LDS adds suffice) and it is written back.
// ---------------------------------------------------------------------------------------------
constexpr int DTILE = 8192;  // floats of dense_out per tile (32 KiB of LDS)
constexpr int DMAXW = 64;    // workers per launch
constexpr int DGROUP = 8;    // workers searched at a time
constexpr int DBATCH = 4;    // pairs per thread and batch
#ifndef GRAVAC_DSPARSE
#define GRAVAC_DSPARSE 512
#endif
constexpr uint32_t DSPARSE = GRAVAC_DSPARSE;   // a tile with at most this many pairs is updated entry by entry
constexpr int DSLOTS = (DSPARSE + 255) / 256;  // pairs per thread of such a tile

struct WorkerOffsets {
    int64_t at[DMAXW + 1];
};

// Both first positions l, h in [a, b) of the ascending array idx with idx[l] >= x0 and idx[h] >= x1
// (x0 <= x1; b if none).  Run by the 32 lanes of one half of a wavefront together; `half` = 0 or 1
// says which half, j = lane within the half.  Each round probes both brackets at once.
__device__ __forceinline__ void lower_bounds_32(const int32_t* idx, int64_t a, int64_t b, int64_t x0, int64_t x1, int half,
                                                int j, int64_t& l, int64_t& h)
{
    int64_t a0 = a, b0 = b, a1 = a, b1 = b;
    bool done0 = false, done1 = false;
    while (!(done0 && done1)) {
        const int64_t n0 = b0 - a0, n1 = b1 - a1;
        const int64_t st0 = n0 > 32 ? (n0 + 31) / 32 : 1, st1 = n1 > 32 ? (n1 + 31) / 32 : 1;
        const int64_t p0 = a0 + (int64_t)j * st0, p1 = a1 + (int64_t)j * st1;
        const bool q0 = !done0 && p0 < b0, q1 = !done1 && p1 < b1;
        const int32_t v0 = q0 ? idx[p0] : 0, v1 = q1 ? idx[p1] : 0;
        const uint32_t c0 = (uint32_t)__popc((uint32_t)(__ballot(q0 && (int64_t)v0 < x0) >> (32 * half)));
        const uint32_t c1 = (uint32_t)__popc((uint32_t)(__ballot(q1 && (int64_t)v1 < x1) >> (32 * half)));
        if (!done0) {
            if (n0 <= 32) { a0 += c0; done0 = true; }            // every position was probed
            else if (c0 == 0) { done0 = true; }                  // idx[a0] >= x0
            else { const int64_t e = a0 + (int64_t)c0 * st0; a0 += (int64_t)(c0 - 1) * st0 + 1; b0 = e < b0 ? e : b0; }
        }
        if (!done1) {
            if (n1 <= 32) { a1 += c1; done1 = true; }
            else if (c1 == 0) { done1 = true; }
            else { const int64_t e = a1 + (int64_t)c1 * st1; a1 += (int64_t)(c1 - 1) * st1 + 1; b1 = e < b1 ? e : b1; }
        }
    }
    l = a0;
    h = a1;
}

__global__ __launch_bounds__(256) void decompress_kernel(const int32_t* __restrict__ idx, const float* __restrict__ val,
                                                         WorkerOffsets wo, int W, int64_t n, float* dense, float alpha)
{
    __shared__ __attribute__((aligned(16))) float acc[DTILE];
    __shared__ int64_t lo[DGROUP], hi[DGROUP];
    __shared__ uint32_t pre[DGROUP + 1];
    __shared__ int32_t first[DMAXW], last[DMAXW];   // smallest and largest index of every worker's message
    const int tid = threadIdx.x;
    const bool vec = (((uintptr_t)dense) & 15) == 0;  // float4 access needs a 16-byte aligned buffer
    if (tid < W) {
        const int64_t a = wo.at[tid], b = wo.at[tid + 1];
        first[tid] = (b > a) ? idx[a] : 0x7FFFFFFF;
        last[tid] = (b > a) ? idx[b - 1] : -1;
    }
    __syncthreads();
    const int64_t ntile = (n + DTILE - 1) / DTILE;
    for (int64_t tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        const int64_t base = tile * DTILE;
        const int len = (int)((n - base < DTILE) ? n - base : DTILE);
        bool loaded = false;
        for (int w0 = 0; w0 < W; w0 += DGROUP) {
            const int wn = (W - w0 < DGROUP) ? W - w0 : DGROUP;
            // can any message of this group touch the tile at all?
            bool maybe = false;
            for (int w = 0; w < wn; ++w)
                maybe |= ((int64_t)first[w0 + w] < base + len) && ((int64_t)last[w0 + w] >= base);
            if (!maybe) continue;
            __syncthreads();  // lo / hi / pre of the previous group or tile are no longer read
            {
                const int w = tid >> 5, j = tid & 31, half = (tid >> 5) & 1;
                // 32 threads per worker; absent workers search an empty range
                const int64_t a = (w < wn) ? wo.at[w0 + w] : 0, b = (w < wn) ? wo.at[w0 + w + 1] : 0;
                int64_t l, h;
                lower_bounds_32(idx, a, b, base, base + len, half, j, l, h);
                if (j == 0 && w < wn) { lo[w] = l; hi[w] = h; }
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t s = 0;
                for (int w = 0; w < DGROUP; ++w) {
                    pre[w] = s;
                    if (w < wn) s += (uint32_t)(hi[w] - lo[w]);
                }
                pre[DGROUP] = s;
            }
            __syncthreads();
            const uint32_t total = pre[DGROUP];
            if (total == 0) continue;  // no message of this group touches the tile
            if (W <= DGROUP && total <= DSPARSE) {
                // few pairs, and this group is all there is: only the entries they name are read and written back (as in
                // the kernel that works from tile boundaries; they still go through the tile buffer, worker by worker)
                int pj[DSLOTS], pw[DSLOTS];
                float pv[DSLOTS], dv[DSLOTS];
                int64_t at[DSLOTS];
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) {
                    const uint32_t slot = q * 256 + tid;
                    const uint32_t sc = slot < total ? slot : total - 1;
                    int w = 0;
#pragma unroll
                    for (int x = 1; x < DGROUP; ++x) w += (sc >= pre[x]);
                    at[q] = lo[w] + (int64_t)(sc - pre[w]);
                    pw[q] = slot < total ? w : -1;
                }
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) pj[q] = idx[at[q]];
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) pv[q] = val[at[q]];
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) {
                    const int64_t j = (int64_t)pj[q] - base;
                    if (j < 0 || j >= len) pw[q] = -1;   // an index outside the tile (malformed message) is ignored
                    pj[q] = (int)(j < 0 || j >= len ? 0 : j);
                }
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) dv[q] = pw[q] >= 0 ? dense[base + pj[q]] : 0.0f;
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q)
                    if (pw[q] >= 0) acc[pj[q]] = dv[q];  // the same value from every pair of that entry
                __syncthreads();
                for (int w = 0; w < wn; ++w) {
                    if (pre[w + 1] == pre[w]) continue;
#pragma unroll
                    for (int q = 0; q < DSLOTS; ++q)
                        if (pw[q] == w) acc[pj[q]] = __fadd_rn(acc[pj[q]], __fmul_rn(alpha, pv[q]));
                    __syncthreads();
                }
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q)
                    if (pw[q] >= 0) dense[base + pj[q]] = acc[pj[q]];
                continue;   // (nothing was loaded whole: nothing is written back; the next tile starts with a barrier)
            }
            if (!loaded) {
                if (vec && len == DTILE) {
                    // a whole tile: all eight loads of a thread in flight together
                    v4f tv[DTILE / 1024];
#pragma unroll
                    for (int r = 0; r < DTILE / 1024; ++r) tv[r] = *(const v4f*)(dense + base + r * 1024 + tid * 4);
#pragma unroll
                    for (int r = 0; r < DTILE / 1024; ++r) *(v4f*)(acc + r * 1024 + tid * 4) = tv[r];
                } else {
                    for (int i = tid * 4; i < len; i += 256 * 4) {
                        if (vec && i + 4 <= len) {
                            const v4f v = *(const v4f*)(dense + base + i);
                            acc[i] = v.x; acc[i + 1] = v.y; acc[i + 2] = v.z; acc[i + 3] = v.w;
                        } else {
                            for (int e = 0; e < 4 && i + e < len; ++e) acc[i + e] = dense[base + i + e];
                        }
                    }
                }
                loaded = true;
            }
            // the group's pairs, worker-major, DBATCH per thread and batch; all loads of a batch in flight together
            for (uint32_t s0 = 0; s0 < total; s0 += 256 * DBATCH) {
                int pj[DBATCH], pw[DBATCH];
                float pv[DBATCH];
                int64_t at[DBATCH];
                // where the pairs lie (a slot past the last pair takes the last pair's place and is not applied:
                // total >= 1 here), then all loads without branches around them, in flight together
#pragma unroll
                for (int q = 0; q < DBATCH; ++q) {
                    const uint32_t slot = s0 + q * 256 + tid;
                    const uint32_t sc = slot < total ? slot : total - 1;
                    int w = 0;
#pragma unroll
                    for (int x = 1; x < DGROUP; ++x) w += (sc >= pre[x]);
                    at[q] = lo[w] + (int64_t)(sc - pre[w]);
                    pw[q] = slot < total ? w : -1;
                }
#pragma unroll
                for (int q = 0; q < DBATCH; ++q) pj[q] = idx[at[q]];
#pragma unroll
                for (int q = 0; q < DBATCH; ++q) pv[q] = val[at[q]];
#pragma unroll
                for (int q = 0; q < DBATCH; ++q) {
                    const int64_t j = (int64_t)pj[q] - base;
                    if (j < 0 || j >= len) pw[q] = -1;   // an index outside the tile (malformed message) is ignored
                    pj[q] = (int)(j < 0 || j >= len ? 0 : j);
                }
                // workers present in this batch: from the worker of its first slot to that of its last
                const uint32_t end = (s0 + 256 * DBATCH < total ? s0 + 256 * DBATCH : total) - 1;
                int wmin = 0, wmax = 0;
#pragma unroll
                for (int x = 1; x < DGROUP; ++x) { wmin += (s0 >= pre[x]); wmax += (end >= pre[x]); }
                __syncthreads();  // tile loaded / previous batch applied
                for (int w = wmin; w <= wmax; ++w) {
#pragma unroll
                    for (int q = 0; q < DBATCH; ++q)
                        if (pw[q] == w) acc[pj[q]] = __fadd_rn(acc[pj[q]], __fmul_rn(alpha, pv[q]));
                    __syncthreads();
                }
            }
        }
        if (loaded) {
            __syncthreads();
            if (vec && len == DTILE) {
#pragma unroll
                for (int r = 0; r < DTILE / 1024; ++r)
                    *(v4f*)(dense + base + r * 1024 + tid * 4) = *(const v4f*)(acc + r * 1024 + tid * 4);
            } else {
                for (int i = tid * 4; i < len; i += 256 * 4) {
                    if (vec && i + 4 <= len) {
                        v4f v;
                        v.x = acc[i]; v.y = acc[i + 1]; v.z = acc[i + 2]; v.w = acc[i + 3];
                        *(v4f*)(dense + base + i) = v;
                    } else {
                        for (int e = 0; e < 4 && i + e < len; ++e) dense[base + i + e] = acc[i + e];
                    }
                }
            }
            __syncthreads();  // the tile buffer is free again
        }
    }
}

// ---------------------------------------------------------------------------------------------
// decompression with a workspace: the tile boundaries of every message are computed once, by one thread
// per pair, instead of being searched for by every tile.
//   bounds[w][t], tile(first index of w) < t <= tile(last index of w): number of pairs of worker w with index
//   below t * DTILE (indices below 0 count as tile 0, indices from ntile * DTILE on as past the last tile).
//   Tile t's pairs of worker w are [bounds[w][t], bounds[w][t + 1]) of its message, where the lower end is 0
//   for the tile of the message's first index and the upper end the message's length for the tile of its last
//   index; entries outside that range are never written and never read.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int64_t tile_of_index(int32_t x, int64_t ntile)
{
    if (x < 0) return 0;
    const int64_t t = (int64_t)x / DTILE;
    return t < ntile ? t : ntile;
}

// grid (pair blocks, workers).  Pair j > 0 of a message starts the tiles (tile of pair j - 1, tile of pair j].
// A lane with up to 2 tiles to write does it itself, longer runs (gaps in the message) are written by the
// whole wavefront.
__global__ __launch_bounds__(256) void bounds_kernel(const int32_t* __restrict__ idx, WorkerOffsets wo, int64_t ntile,
                                                     uint32_t* __restrict__ bounds)
{
    const int w = blockIdx.y, lane = threadIdx.x & 63;
    const int64_t a = wo.at[w], cnt = wo.at[w + 1] - a;
    uint32_t* bw = bounds + (size_t)w * (size_t)(ntile + 1);
    const int64_t j0 = ((int64_t)blockIdx.x * 256 + (threadIdx.x & ~63));  // first pair of this wavefront
    if (j0 >= cnt) return;
    const int64_t j = j0 + lane;
    const bool live = j > 0 && j < cnt;
    int64_t t_prev = 0, t_cur = 0;  // this lane writes bw[t] = j for t in (t_prev, t_cur]
    if (live) {
        t_cur = tile_of_index(idx[a + j], ntile);
        t_prev = tile_of_index(idx[a + j - 1], ntile);
    }
    const int64_t gap = t_cur - t_prev;  // <= 0 where the indices do not ascend: nothing is written
    if (live && gap > 0 && gap <= 2) {
        bw[t_prev + 1] = (uint32_t)j;
        if (gap == 2) bw[t_prev + 2] = (uint32_t)j;
    }
    uint64_t big = __ballot(live && gap > 2);
    while (big) {
        const int src = __ffsll((unsigned long long)big) - 1;
        big &= big - 1;
        const int64_t tp = __shfl(t_prev, src, 64), tc = __shfl(t_cur, src, 64);
        const uint32_t v = (uint32_t)(j0 + src);
        for (int64_t t = tp + 1 + lane; t <= tc; t += 64) bw[t] = v;
    }
}

constexpr int DCHUNK = 32;  // tiles whose boundaries a workgroup fetches in one round of loads
constexpr int DENT = 768;   // (tile, worker) entries of such a chunk

// A workgroup takes the tiles blockIdx.x, blockIdx.x + gridDim.x, ...  It first fetches, for a chunk of its
// tiles at once, every worker's boundaries (one round of independent loads instead of one dependent round per
// tile) and then walks over the chunk's tiles; a tile no message has a pair in costs no further memory access.
__global__ __launch_bounds__(256) void decompress_ws_kernel(const int32_t* __restrict__ idx, const float* __restrict__ val,
                                                            WorkerOffsets wo, int W, int64_t n, float* dense,
                                                            const uint32_t* __restrict__ bounds, float alpha)
{
    __shared__ __attribute__((aligned(16))) float acc[DTILE];
    __shared__ uint32_t blo[DENT], bcnt[DENT];      // first pair and number of pairs, per (tile of the chunk, worker)
    __shared__ uint32_t btot[DCHUNK];               // pairs of all workers, per tile of the chunk
    __shared__ uint32_t spre[DMAXW + 1];            // a sparse tile's pairs before worker w, in worker-major order
    __shared__ int64_t wat[DMAXW + 1];              // start of every worker's message
    __shared__ int32_t first[DMAXW], last[DMAXW];   // smallest and largest index of every worker's message
    const int tid = threadIdx.x;
    const bool vec = (((uintptr_t)dense) & 15) == 0;  // float4 access needs a 16-byte aligned buffer
    if (tid <= DMAXW) wat[tid] = wo.at[tid];
    if (tid < W) {
        const int64_t a = wo.at[tid], b = wo.at[tid + 1];
        first[tid] = (b > a) ? idx[a] : 0x7FFFFFFF;
        last[tid] = (b > a) ? idx[b - 1] : -1;
    }
    const int64_t ntile = (n + DTILE - 1) / DTILE;
    const int Wp = (W + DGROUP - 1) / DGROUP * DGROUP;            // workers, padded to whole groups
    const int tc = DENT / Wp < DCHUNK ? DENT / Wp : DCHUNK;       // tiles per chunk (>= 12: Wp <= 64)
    for (int64_t c0 = blockIdx.x; c0 < ntile; c0 += (int64_t)tc * gridDim.x) {
        __syncthreads();  // first / last / wat are written; the previous chunk's entries are no longer read
        if (tid < DCHUNK) btot[tid] = 0;
        __syncthreads();
        for (int e = tid; e < tc * Wp; e += 256) {
            const int i = e / Wp, w = e - i * Wp;
            const int64_t tile = c0 + (int64_t)i * gridDim.x;
            uint32_t l = 0, c = 0;
            if (w < W && tile < ntile) {
                const int64_t base = tile * DTILE, end = (n - base < DTILE) ? n : base + DTILE;
                if ((int64_t)first[w] < end && (int64_t)last[w] >= base) {
                    const uint32_t* bw = bounds + (size_t)w * (size_t)(ntile + 1) + tile;
                    const uint32_t cw = (uint32_t)(wat[w + 1] - wat[w]);
                    uint32_t h = cw;
                    if (tile > tile_of_index(first[w], ntile)) l = bw[0];
                    if (tile < tile_of_index(last[w], ntile)) h = bw[1];
                    // clamped to the message, so that no read can leave it even if the indices were not ascending
                    l = l < cw ? l : cw;
                    h = h < l ? l : (h < cw ? h : cw);
                    c = h - l;
                }
            }
            blo[e] = l;
            bcnt[e] = c;
            if (c) atomicAdd(&btot[i], c);
        }
        __syncthreads();
        for (int i = 0; i < tc; ++i) {
            const int64_t tile = c0 + (int64_t)i * gridDim.x;
            if (tile >= ntile) break;
            const int64_t base = tile * DTILE;
            const int len = (int)((n - base < DTILE) ? n - base : DTILE);
            const uint32_t tot = btot[i];
            if (tot == 0) continue;  // no message touches the tile
            if (tot <= DSPARSE) {
                // Few pairs: only the entries they name are read and written back, not the whole tile (a scattered
                // access moves 64 bytes, so this pays up to about one pair per 16 entries).  The entries go through
                // the tile buffer all the same, so that pairs of different workers with the same index are added in
                // worker order.
                if (tid < 64) {
                    const uint32_t inc = wave_scan(tid < Wp ? bcnt[i * Wp + tid] : 0u);
                    spre[tid + 1] = inc;
                    if (tid == 0) spre[0] = 0;
                }
                __syncthreads();
                int pj[DSLOTS], pw[DSLOTS];
                float pv[DSLOTS], dv[DSLOTS];
                int64_t at[DSLOTS];
                // the tile's pairs in worker-major order, DSLOTS per thread (a slot past the last pair takes the last
                // pair's place and is not applied)
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) {
                    const uint32_t slot = q * 256 + tid;
                    const uint32_t sc = slot < tot ? slot : tot - 1;
                    int w = 0;
#pragma unroll
                    for (int step = 32; step >= 1; step >>= 1)
                        if (spre[w + step] <= sc) w += step;   // spre[64] = tot > sc: w stays below 64
                    at[q] = wat[w] + (int64_t)blo[i * Wp + w] + (int64_t)(sc - spre[w]);
                    pw[q] = slot < tot ? w : -1;
                }
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) pj[q] = idx[at[q]];
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) pv[q] = val[at[q]];
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) {
                    const int64_t j = (int64_t)pj[q] - base;
                    if (j < 0 || j >= len) pw[q] = -1;   // an index outside the tile (malformed message) is ignored
                    pj[q] = (int)(j < 0 || j >= len ? 0 : j);
                }
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q) dv[q] = pw[q] >= 0 ? dense[base + pj[q]] : 0.0f;
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q)
                    if (pw[q] >= 0) acc[pj[q]] = dv[q];  // the same value from every pair of that entry
                __syncthreads();
                for (int w = 0; w < W; ++w) {
                    if (bcnt[i * Wp + w] == 0) continue;
#pragma unroll
                    for (int q = 0; q < DSLOTS; ++q)
                        if (pw[q] == w) acc[pj[q]] = __fadd_rn(acc[pj[q]], __fmul_rn(alpha, pv[q]));
                    __syncthreads();
                }
#pragma unroll
                for (int q = 0; q < DSLOTS; ++q)
                    if (pw[q] >= 0) dense[base + pj[q]] = acc[pj[q]];
                __syncthreads();  // the tile buffer and spre are free again
                continue;
            }
            bool loaded = false;
            for (int w0 = 0; w0 < W; w0 += DGROUP) {
                const uint32_t* cg = bcnt + i * Wp + w0;
                const uint32_t* lg = blo + i * Wp + w0;
                uint32_t pre[DGROUP + 1];
                pre[0] = 0;
#pragma unroll
                for (int w = 0; w < DGROUP; ++w) pre[w + 1] = pre[w] + cg[w];
                const uint32_t total = pre[DGROUP];
                if (total == 0) continue;  // no message of this group touches the tile
                if (!loaded) {
                    if (vec && len == DTILE) {
                        // a whole tile: all eight loads of a thread in flight together
                        v4f tv[DTILE / 1024];
#pragma unroll
                        for (int r = 0; r < DTILE / 1024; ++r) tv[r] = *(const v4f*)(dense + base + r * 1024 + tid * 4);
#pragma unroll
                        for (int r = 0; r < DTILE / 1024; ++r) *(v4f*)(acc + r * 1024 + tid * 4) = tv[r];
                    } else {
                        for (int q = tid * 4; q < len; q += 256 * 4) {
                            if (vec && q + 4 <= len) {
                                const v4f v = *(const v4f*)(dense + base + q);
                                acc[q] = v.x; acc[q + 1] = v.y; acc[q + 2] = v.z; acc[q + 3] = v.w;
                            } else {
                                for (int e = 0; e < 4 && q + e < len; ++e) acc[q + e] = dense[base + q + e];
                            }
                        }
                    }
                    loaded = true;
                }
                // the group's pairs, worker-major, DBATCH per thread and batch; all loads of a batch in flight together
                for (uint32_t s0 = 0; s0 < total; s0 += 256 * DBATCH) {
                    int pj[DBATCH], pw[DBATCH];
                    float pv[DBATCH];
                    int64_t at[DBATCH];
                    // where the pairs lie (a slot past the last pair takes the last pair's place and is not applied:
                    // total >= 1 here), then all loads without branches around them, in flight together
#pragma unroll
                    for (int q = 0; q < DBATCH; ++q) {
                        const uint32_t slot = s0 + q * 256 + tid;
                        const uint32_t sc = slot < total ? slot : total - 1;
                        int w = 0;
#pragma unroll
                        for (int x = 1; x < DGROUP; ++x) w += (sc >= pre[x]);
                        uint32_t pb = 0;
#pragma unroll
                        for (int x = 1; x < DGROUP; ++x) if (x == w) pb = pre[x];
                        at[q] = wat[w0 + w] + (int64_t)lg[w] + (int64_t)(sc - pb);
                        pw[q] = slot < total ? w : -1;
                    }
#pragma unroll
                    for (int q = 0; q < DBATCH; ++q) pj[q] = idx[at[q]];
#pragma unroll
                    for (int q = 0; q < DBATCH; ++q) pv[q] = val[at[q]];
#pragma unroll
                    for (int q = 0; q < DBATCH; ++q) {
                        const int64_t j = (int64_t)pj[q] - base;
                        if (j < 0 || j >= len) pw[q] = -1;   // an index outside the tile (malformed message) is ignored
                        pj[q] = (int)(j < 0 || j >= len ? 0 : j);
                    }
                    // workers present in this batch: from the worker of its first slot to that of its last
                    const uint32_t end = (s0 + 256 * DBATCH < total ? s0 + 256 * DBATCH : total) - 1;
                    int wmin = 0, wmax = 0;
#pragma unroll
                    for (int x = 1; x < DGROUP; ++x) { wmin += (s0 >= pre[x]); wmax += (end >= pre[x]); }
                    __syncthreads();  // tile loaded / previous batch applied
                    for (int w = wmin; w <= wmax; ++w) {
#pragma unroll
                        for (int q = 0; q < DBATCH; ++q)
                            if (pw[q] == w) acc[pj[q]] = __fadd_rn(acc[pj[q]], __fmul_rn(alpha, pv[q]));
                        __syncthreads();
                    }
                }
            }
            if (loaded) {
                __syncthreads();
                if (vec && len == DTILE) {
#pragma unroll
                    for (int r = 0; r < DTILE / 1024; ++r)
                        *(v4f*)(dense + base + r * 1024 + tid * 4) = *(const v4f*)(acc + r * 1024 + tid * 4);
                } else {
                    for (int q = tid * 4; q < len; q += 256 * 4) {
                        if (vec && q + 4 <= len) {
                            v4f v;
                            v.x = acc[q]; v.y = acc[q + 1]; v.z = acc[q + 2]; v.w = acc[q + 3];
                            *(v4f*)(dense + base + q) = v;
                        } else {
                            for (int e = 0; e < 4 && q + e < len; ++e) dense[base + q + e] = acc[q + e];
                        }
                    }
                }
                __syncthreads();  // the tile buffer is free again
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// A layerwise call's tables, from the pinned host buffer they were built in into the workspace.  A kernel that
// reads the host buffer is queued like every other kernel of the call; a copy by the DMA engine starts 10 to 20 us
// later and the call's first kernel waits for it.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void table_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, uint32_t n16)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------
// Commit of a message: residual[idx[i]] = +0.0f.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void commit_kernel(const int32_t* __restrict__ idx, int64_t count,
                                                     float* __restrict__ residual, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const int64_t g = idx[i];
        if ((uint64_t)g < (uint64_t)n) residual[g] = 0.0f;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t status, tables, tables_bytes, tseg, st, seg, bnd_lo, bnd_hi, bnd_mid, hist1, ovfc, hist2, coarse, list_key, list_tile,
        list_val, list_cnt, samp_hist, samp_grp, cand_cnt, brk_cnt, ovn, ovs, tg0, tin, toff, ttake, tsel, ssd, ssd_t, sss,
        cand_idx, cand_val, brk_key, brk_val, total;
};

// Upper bounds that depend only on (n, n_seg).
uint64_t max_tiles(int64_t n, int n_seg) { return (uint64_t)((n + TW - 1) / TW) + (uint64_t)n_seg; }

uint64_t max_sample_blocks(int64_t n, int n_seg)
{
    static_assert(DENSE_BLOCKS * SAMPLE_BLOCK <= 2 * SAMPLE_MAX && SAMPLE_MAX_FLAT <= DENSE_BLOCKS * SAMPLE_BLOCK * DENSE_ROUNDS,
                  "the blocks of a dense sample fit as well");
    const uint64_t a = (uint64_t)n_seg * (2 * (n_seg > 1 ? SAMPLE_MAX_SEG : SAMPLE_MAX) / SAMPLE_BLOCK);
    const uint64_t b = (uint64_t)((n + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK) + (uint64_t)n_seg;
    return a < b ? a : b;
}

// Copy blocks of the bracket histograms and gather lists.  Global atomics on one cache line queue up, so a large
// tensor spreads them over REP copies (with one copy the streaming pass of the 314-tensor ResNet list takes 120
// instead of 97 us); a small tensor puts so few entries into its brackets that fewer do: 1 below 2^17 elements, then
// 2, 4 and from 2^19 elements on REP.  A flat call always takes REP.  A tensor's copies number at most
// 1 + nt / 2^16, which bounds a layerwise call's total by n_seg + n / 2^16.
uint32_t seg_copies(int64_t nt, bool flat)
{
    static_assert(REP == 8, "1, 2, 4, 8 copies");
    if (flat || nt >= (1 << 19)) return REP;
    return nt >= (1 << 18) ? 4u : nt >= (1 << 17) ? 2u : 1u;
}
size_t pool_blocks(int64_t n, int n_cf, int n_seg)
{
    if (n_seg <= 1) return (size_t)n_cf * REP;
    const size_t graded = (size_t)n_seg + (size_t)(n >> 16), all = (size_t)n_seg * REP;
    return (size_t)n_cf * (graded < all ? graded : all);
}

Layout make_layout(int64_t n, int n_cf, int n_seg)
{
    Layout L;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
    const uint64_t nt = max_tiles(n, n_seg), nsb = max_sample_blocks(n, n_seg);
    const size_t sc = (size_t)n_seg * n_cf;
    L.status = take(sizeof(Status));
    // host-built tables, one piece: SegInfo[n_seg], ktab[n_seg][n_cf], sblock_seg[sample blocks], small_list[n_seg]
    L.tables_bytes = sizeof(SegInfo) * n_seg + sizeof(uint32_t) * sc + sizeof(uint32_t) * nsb + sizeof(uint32_t) * n_seg;
    L.tables = take(L.tables_bytes);
    L.tseg = take(sizeof(uint32_t) * nt);
    L.st = take(sizeof(CfState) * sc);
    L.seg = take(sizeof(SegState) * n_seg);
    L.bnd_lo = take(sizeof(uint32_t) * sc);
    L.bnd_hi = take(sizeof(uint32_t) * sc);
    L.bnd_mid = take(sizeof(uint32_t) * sc);
    const size_t blocks = pool_blocks(n, n_cf, n_seg);
    L.hist1 = take(sizeof(uint32_t) * blocks * NBIN);
    L.ovfc = take(sizeof(uint32_t) * sc * 64 * 32);
    L.hist2 = take(sizeof(uint32_t) * sc * NBIN);
    L.coarse = take(sizeof(uint32_t) * (size_t)n_seg * NBIN);
    L.list_key = take(sizeof(uint32_t) * blocks * LCAP);
    L.list_tile = take(sizeof(uint32_t) * blocks * LCAP);
    L.list_val = take(sizeof(float) * blocks * LCAP);
    L.list_cnt = take(sizeof(uint32_t) * blocks * 32);
    L.samp_hist = take(sizeof(uint32_t) * nsb * (SBIN / 2));
    L.samp_grp = take(sizeof(uint32_t) * nsb * SGRP);
    L.cand_cnt = take(sizeof(uint32_t) * nt * SUB);
    L.brk_cnt = take(sizeof(uint32_t) * nt * SUB);
    L.ovn = take(sizeof(uint32_t) * nt * SUB * n_cf);
    L.ovs = take(sizeof(double) * nt * SUB * n_cf);
    L.tg0 = take(sizeof(uint32_t) * nt);
    L.tin = take(sizeof(uint32_t) * nt);
    L.toff = take(sizeof(uint32_t) * nt);
    L.ttake = take(sizeof(uint32_t) * nt);
    L.tsel = take(sizeof(uint32_t) * nt);
    L.ssd = take(sizeof(double) * nt * SUB);
    L.ssd_t = take(sizeof(double) * nt);
    L.sss = take(sizeof(double) * nt * n_cf);
    L.cand_idx = take(sizeof(int32_t) * nt * TW);
    L.cand_val = take(sizeof(float) * nt * TW);
    L.brk_key = take(sizeof(uint32_t) * nt * TW);
    L.brk_val = take(sizeof(float) * nt * TW);
    L.total = at;
    return L;
}

// samples taken from a segment of nt elements when the CFs range from cf_min to cf_max
uint32_t sample_count(uint64_t nt, double cf_min, double cf_max, bool flat)
{
    // layerwise: the larger of 32 CF_max and 1/64 of the tensor.  A small sample of a large tensor gives a wide
    // bracket: many more entries in it than k, and bins so coarse that the keys near the bracket's lower end crowd
    // into a few histogram bins, where their atomics queue up behind each other
    uint64_t target = flat ? (uint64_t)SAMPLE_MAX : (uint64_t)(32.0 * std::ceil(cf_max));
    if (!flat && target < nt / 64) target = nt / 64;
    if (target < 4096) target = 4096;
    const uint64_t cap = flat ? SAMPLE_MAX : SAMPLE_MAX_SEG;
    if (target > cap) target = cap;
    if (flat) {
        // The bracket spans about 10 standard deviations of a sampled rank, which is 10 sqrt(k nt / m) of the tensor's
        // entries for m samples, and every entry inside it costs the streaming pass a device-wide atomic (about
        // ten per nanosecond all told, and a gradient whose large entries sit together sends them all at once): a
        // selection of many entries from a large tensor (k = nt / cf_min) takes more samples, enough to keep that
        // number near 300,000.
        const double need = 64.0 * ((double)nt / cf_min) * (double)nt / 68719476736.0;  // 2^36
        if (need > (double)target) target = need > (double)SAMPLE_MAX_FLAT ? (uint64_t)SAMPLE_MAX_FLAT : (uint64_t)need;
    }
    const uint64_t unit = target > (uint64_t)SAMPLE_MAX ? SAMPLE_BLOCK * DENSE_ROUNDS : SAMPLE_BLOCK;
    target = (target + unit - 1) / unit * unit;
    return (nt <= 2 * target) ? (uint32_t)nt : (uint32_t)target;
}

// Pinned host staging for the layerwise tables: a small ring of slots, each followed on its stream by an
// event, so that a slot is only rewritten after the copy that read it has run.  Host memory only; grown on demand.
// This ring is the only state the library keeps between calls.
struct StagingSlot {
    char* mem = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool pending = false;  // `done` was recorded and not yet waited for
    bool busy = false;     // held by a caller (being waited for, filled or copied from)
};
constexpr int STAGING_SLOTS = 8;
StagingSlot g_staging[STAGING_SLOTS];
int g_staging_next = 0;
std::mutex g_staging_mutex;

StagingSlot* staging_acquire(size_t bytes)
{
    StagingSlot* s = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_staging_mutex);
        // A slot that is large enough and whose last copy has run; else, while fewer than two slots have memory, one
        // without (it is allocated below); else one whose copy is still queued (its event is waited for below: the host
        // then runs at most a call or two ahead of the GPU); else, all of those being held by other callers, one
        // without memory.  Pinning fresh host memory takes milliseconds and slows the first copy out of it, so a caller
        // that runs ahead of the GPU does not get a new slot for every call it is ahead.
        int with_mem = 0;
        for (int i = 0; i < STAGING_SLOTS; ++i) with_mem += g_staging[i].cap > 0 ? 1 : 0;
        for (int pass = 0; pass < 4 && !s; ++pass) {
            if (pass == 1 && with_mem >= 2) continue;
            for (int i = 0; i < STAGING_SLOTS && !s; ++i) {
                StagingSlot* c = &g_staging[(g_staging_next + i) % STAGING_SLOTS];
                if (c->busy) continue;
                const bool ready = c->cap >= bytes && (!c->pending || hipEventQuery(c->done) == hipSuccess);
                if ((pass == 0 && ready) || ((pass == 1 || pass == 3) && c->cap == 0) || (pass == 2 && c->cap > 0)) {
                    s = c;
                    g_staging_next = (g_staging_next + i + 1) % STAGING_SLOTS;
                }
            }
        }
        if (!s) return nullptr;  // more concurrent callers than slots
        s->busy = true;
    }
    // the slot is this caller's now: the waiting and the allocation happen outside the lock
    bool ok = true;
    if (!s->done && hipEventCreateWithFlags(&s->done, hipEventDisableTiming) != hipSuccess) { s->done = nullptr; ok = false; }
    if (ok && s->pending) {
        if (hipEventSynchronize(s->done) != hipSuccess) ok = false;
        else s->pending = false;
    }
    if (ok && s->cap < bytes) {
        if (s->mem) (void)hipHostFree(s->mem);
        s->mem = nullptr; s->cap = 0;
        const size_t want = bytes < 65536 ? 65536 : bytes + bytes / 2;
        if (hipHostMalloc((void**)&s->mem, want, hipHostMallocDefault) != hipSuccess) { s->mem = nullptr; ok = false; }
        else s->cap = want;
    }
    if (!ok) {
        std::lock_guard<std::mutex> lock(g_staging_mutex);
        s->busy = false;
        return nullptr;
    }
    return s;
}

void staging_release(StagingSlot* s, bool recorded)
{
    std::lock_guard<std::mutex> lock(g_staging_mutex);
    s->pending = recorded;
    s->busy = false;
}

}  // namespace

// Scratch of gravac_decompress_accumulate_static, the entry point for callers that cannot allocate: the tile
// boundaries of the messages (what the caller's workspace holds in gravac_decompress_accumulate).  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returned.
constexpr size_t STATIC_SCRATCH_WORDS = (size_t)GRAVAC_STATIC_SCRATCH_BYTES / sizeof(uint32_t);
static __device__ __align__(256) uint32_t scratch[STATIC_SCRATCH_WORDS];

namespace {

constexpr int MAX_DEVICES = 64;
uint32_t* g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on every device used so far
std::mutex g_scratch_mutex;

// The address of `scratch` on the current device, looked up once per device.
int static_scratch(uint32_t** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return GRAVAC_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return GRAVAC_ERR_HIP;
        g_scratch_ptr[dev] = (uint32_t*)ptr;
    }
    *out = g_scratch_ptr[dev];
    return GRAVAC_OK;
}

}  // namespace

extern "C" {

int64_t gravac_topk_count(int64_t n, double cf)
{
    if (n <= 0 || !(cf >= 1.0) || std::isinf(cf)) return -1;
    int64_t k;
    if (cf == std::floor(cf) && cf < 9.0e18) {
        const int64_t c = (int64_t)cf;
        k = (n + c - 1) / c;
    } else {
        k = (int64_t)std::ceil((double)n / cf);
    }
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

int gravac_workspace_bytes(int64_t n, int n_cf, int n_seg, size_t* bytes_out)
{
    if (!bytes_out || n <= 0 || n > 2147483647LL || n_cf < 1 || n_cf > MAXCF || n_seg < 0) return GRAVAC_ERR_INVALID_ARG;
    if ((int64_t)n_seg > n) return GRAVAC_ERR_INVALID_ARG;
    *bytes_out = make_layout(n, n_cf, n_seg < 1 ? 1 : n_seg).total;
    return GRAVAC_OK;
}

// GRAVAC_OK if `stream` is not being captured into a graph, else GRAVAC_ERR_CAPTURE (asked only by calls that cannot
// be replayed: a replay would copy whatever the staging slot holds by then, or re-record the caller's events).
static int refuse_capture(hipStream_t stream)
{
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) return GRAVAC_ERR_HIP;
    return cap == hipStreamCaptureStatusNone ? GRAVAC_OK : GRAVAC_ERR_CAPTURE;
}

// The pipeline behind all compression entry points.  map_idx == null: error-feedback compression of grad + residual.
// map_idx != null: single-source mode, the source is grad alone (a message's values), map_idx its indices,
// restore / n_restore the dense residual that takes the unselected values back (may be null).
// seed != null: Random-k.  ev != null: the caller's events are recorded around the call and the pass over the gradient.
static int compress_impl(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                         const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val, int64_t out_capacity,
                         int64_t* out_count, double* out_stats, void* workspace, size_t workspace_bytes, unsigned flags,
                         hipStream_t stream, const int32_t* map_idx, float* restore, int64_t n_restore,
                         const uint64_t* seed, const gravac_profile_events* ev, const float* tau = nullptr)
{
    const bool single = map_idx != nullptr;
    const bool random = seed != nullptr;
    const bool fixed = tau != nullptr;  // the threshold sparsifier: one flat tensor, cf_list = {1}, out_capacity as given
    if (fixed && (single || random || n_seg != 0 || n_cf != 1 || !out_count || out_capacity < 0)) return GRAVAC_ERR_INVALID_ARG;
    if (fixed && (!(*tau > 0.0f) || std::isinf(*tau))) return GRAVAC_ERR_INVALID_ARG;
    if (!grad || (!single && !residual) || !cf_list || !out_stats) return GRAVAC_ERR_INVALID_ARG;
    if ((!out_idx || !out_val) && !(fixed && out_capacity == 0)) return GRAVAC_ERR_INVALID_ARG;
    if (n <= 0 || n > 2147483647LL || n_cf < 1 || n_cf > MAXCF || commit < 0 || commit >= n_cf) return GRAVAC_ERR_INVALID_ARG;
    if (((uintptr_t)grad & 3) || ((uintptr_t)residual & 3) || ((uintptr_t)map_idx & 3)) return GRAVAC_ERR_INVALID_ARG;
    if (flags & ~(unsigned)(GRAVAC_FLAG_FORCE_FALLBACK | GRAVAC_FLAG_NO_COMMIT)) return GRAVAC_ERR_INVALID_ARG;
    if ((flags & GRAVAC_FLAG_NO_COMMIT) && (single || fixed)) return GRAVAC_ERR_INVALID_ARG;
    if (n_seg < 0 || (n_seg > 0 && !seg_offsets) || (int64_t)n_seg > n) return GRAVAC_ERR_INVALID_ARG;
    if (ev && (!ev->call_begin || !ev->pass_begin || !ev->pass_end || !ev->call_end)) return GRAVAC_ERR_INVALID_ARG;
    double cf_max = 1.0, cf_min = cf_list[0];
    for (int j = 0; j < n_cf; ++j) {
        if (!(cf_list[j] >= 1.0) || std::isinf(cf_list[j])) return GRAVAC_ERR_INVALID_ARG;
        if (cf_list[j] > cf_max) cf_max = cf_list[j];
        if (cf_list[j] < cf_min) cf_min = cf_list[j];
    }
    const int ns = n_seg < 1 ? 1 : n_seg;
    if (n_seg >= 1) {
        if (seg_offsets[0] != 0 || seg_offsets[n_seg] != n) return GRAVAC_ERR_INVALID_ARG;
        for (int t = 0; t < n_seg; ++t)
            if (seg_offsets[t + 1] <= seg_offsets[t]) return GRAVAC_ERR_INVALID_ARG;
    }
    if (!workspace || ((uintptr_t)workspace & 255)) return GRAVAC_ERR_WORKSPACE;
    const Layout L = make_layout(n, n_cf, ns);
    if (workspace_bytes < L.total) return GRAVAC_ERR_WORKSPACE;

    char* ws = (char*)workspace;
    Params p;
    std::memset(&p, 0, sizeof(p));
    p.grad = grad; p.res = residual; p.acc = single ? grad : residual;
    p.map_idx = map_idx; p.restore = restore; p.n_restore = restore ? n_restore : 0; p.single = single ? 1 : 0;
    // 16-byte accesses need 16-byte aligned buffers; anything else is read and written element by element
    p.vec_ok = (((uintptr_t)grad & 15) == 0 && ((uintptr_t)residual & 15) == 0 && ((uintptr_t)map_idx & 15) == 0) ? 1 : 0;
    p.split = (cf_list[commit] > cf_min) ? 1 : 0;
    p.no_commit = (flags & GRAVAC_FLAG_NO_COMMIT) ? 1 : 0;
    p.bounds_from = (flags & GRAVAC_FLAG_FORCE_FALLBACK) ? BOUNDS_FORCED : (random ? BOUNDS_RANDOM : BOUNDS_SAMPLED);
    if (fixed) {
        p.bounds_from = BOUNDS_FIXED;
        std::memcpy(&p.fixed_key, tau, sizeof(uint32_t));   // positive and finite: the bit pattern is the key
    }
    if (random) {
        // the seed goes through SplitMix64 (its first output for that seed) and gives the two 31-bit keys
        uint64_t z = *seed + 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        p.random = 1;
        p.rk_s0 = (uint32_t)(z & 0x7FFFFFFFull);
        p.rk_s1 = (uint32_t)((z >> 32) & 0x7FFFFFFFull);
    }
    p.n = n; p.n_seg = ns; p.n_cf = n_cf; p.commit = commit;
    p.status = (Status*)(ws + L.status);
    p.segs = (const SegInfo*)(ws + L.tables);
    p.ktab = (const uint32_t*)(ws + L.tables + sizeof(SegInfo) * ns);
    p.sblock_seg = p.ktab + (size_t)ns * n_cf;
    p.tseg = (uint32_t*)(ws + L.tseg);
    p.st = (CfState*)(ws + L.st);
    p.seg = (SegState*)(ws + L.seg);
    p.bnd_lo = (uint32_t*)(ws + L.bnd_lo);
    p.bnd_hi = (uint32_t*)(ws + L.bnd_hi);
    p.bnd_mid = (uint32_t*)(ws + L.bnd_mid);
    p.hist1 = (uint32_t*)(ws + L.hist1);
    p.ovfc = (uint32_t*)(ws + L.ovfc);
    p.hist2 = (uint32_t*)(ws + L.hist2);
    p.coarse = (uint32_t*)(ws + L.coarse);
    p.list_key = (uint32_t*)(ws + L.list_key);
    p.list_tile = (uint32_t*)(ws + L.list_tile);
    p.list_val = (float*)(ws + L.list_val);
    p.list_cnt = (uint32_t*)(ws + L.list_cnt);
    p.samp_hist = (uint32_t*)(ws + L.samp_hist);
    p.samp_grp = (uint32_t*)(ws + L.samp_grp);
    p.cand_cnt = (uint32_t*)(ws + L.cand_cnt);
    p.brk_cnt = (uint32_t*)(ws + L.brk_cnt);
    p.ovn = (uint32_t*)(ws + L.ovn);
    p.ovs = (double*)(ws + L.ovs);
    p.tg0 = (uint32_t*)(ws + L.tg0);
    p.tin = (uint32_t*)(ws + L.tin);
    p.toff = (uint32_t*)(ws + L.toff);
    p.ttake = (uint32_t*)(ws + L.ttake);
    p.tsel = (uint32_t*)(ws + L.tsel);
    p.ssd = (double*)(ws + L.ssd);
    p.ssd_t = (double*)(ws + L.ssd_t);
    p.sss = (double*)(ws + L.sss);
    p.cand_idx = (int32_t*)(ws + L.cand_idx);
    p.cand_val = (float*)(ws + L.cand_val);
    p.brk_key = (uint32_t*)(ws + L.brk_key);
    p.brk_val = (float*)(ws + L.brk_val);
    p.out_idx = out_idx; p.out_val = out_val; p.out_count = out_count; p.out_stats = out_stats;

    int64_t total_out = 0;
    uint32_t max_seg_tiles = 1;  // tiles of the largest segment
    int sample_rounds = 1;       // groups per thread of the sampling kernel
    uint32_t n_small = 0;        // layerwise: tensors of at most SMALL_MAX elements, one workgroup each (not under the
                                 // testing flag, which sends every tensor through the histogram route)
    const bool small_ok = ns > 1 && !(flags & GRAVAC_FLAG_FORCE_FALLBACK);
    StagingSlot* slot = nullptr;
    size_t table_bytes = 0;
    if (ns == 1) {
        for (int j = 0; j < n_cf; ++j) p.flat_k[j] = (uint32_t)gravac_topk_count(n, cf_list[j]);
        p.flat_samples = sample_count((uint64_t)n, cf_min, cf_max, true);
        p.n_tiles = (uint32_t)((n + TW - 1) / TW);
        max_seg_tiles = p.n_tiles;
        // more than SAMPLE_MAX samples (never a tensor read whole): 2 or 4 times SAMPLE_BLOCK samples per block, the
        // fewest that leave at most DENSE_BLOCKS blocks (more blocks keep more loads in flight, fewer cost the
        // threshold kernel less)
        if (p.flat_samples > (uint32_t)SAMPLE_MAX && (int64_t)p.flat_samples != n)
            while (sample_rounds < DENSE_ROUNDS && p.flat_samples > (uint32_t)(DENSE_BLOCKS * SAMPLE_BLOCK * sample_rounds))
                sample_rounds *= 2;
        const uint32_t per_block = SAMPLE_BLOCK * sample_rounds;
        p.n_sample_blocks = (p.flat_samples + per_block - 1) / per_block;
        total_out = p.flat_k[commit];
        if (fixed) {
            // the number of pairs is only known on the device: the emit step writes up to the caller's capacity
            total_out = out_capacity < n ? out_capacity : n;
            p.flat_k[0] = (uint32_t)total_out;
        }
        if (total_out > out_capacity) return GRAVAC_ERR_CAPACITY;
    } else {
        // layerwise tables: sized first, then built straight into a pinned staging slot and copied into the
        // workspace with one asynchronous copy (no host synchronisation)
        uint64_t tiles = 0, sblocks = 0;
        for (int t = 0; t < ns; ++t) {
            const int64_t nt = seg_offsets[t + 1] - seg_offsets[t];
            total_out += gravac_topk_count(nt, cf_list[commit]);
            if (small_ok && nt <= SMALL_MAX) { ++n_small; continue; }  // one workgroup does it all: no tiles, no samples
            const uint64_t tt = (uint64_t)((nt + TW - 1) / TW);
            tiles += tt;
            if (tt > max_seg_tiles) max_seg_tiles = (uint32_t)tt;
            sblocks += (sample_count((uint64_t)nt, cf_min, cf_max, false) + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
        }
        if (total_out > out_capacity) return GRAVAC_ERR_CAPACITY;
        if (tiles > max_tiles(n, ns) || sblocks > max_sample_blocks(n, ns)) return GRAVAC_ERR_WORKSPACE;
        p.n_tiles = (uint32_t)tiles;
        p.n_sample_blocks = (uint32_t)sblocks;
    }
    // nothing has been queued or written up to here; from here on an error return leaves the outputs unspecified
    if (ns > 1 || ev)
        if (const int rc = refuse_capture(stream)) return rc;
    (void)hipGetLastError();  // an error left behind by earlier work of the process is not this call's
    if (ns > 1) {
        table_bytes = sizeof(SegInfo) * ns + sizeof(uint32_t) * (size_t)ns * n_cf + sizeof(uint32_t) * p.n_sample_blocks +
                      sizeof(uint32_t) * n_small;
        table_bytes = (table_bytes + 15) & ~(size_t)15;   // (moved 16 bytes at a time; the workspace's part is that long)
        slot = staging_acquire(table_bytes);
        if (!slot) return GRAVAC_ERR_HIP;
        SegInfo* segs = (SegInfo*)slot->mem;
        uint32_t* ktab = (uint32_t*)(slot->mem + sizeof(SegInfo) * ns);
        uint32_t* sblock_seg = ktab + (size_t)ns * n_cf;
        uint32_t* small_list = sblock_seg + p.n_sample_blocks;
        p.small_list = p.sblock_seg + p.n_sample_blocks;
        p.n_small = n_small;
        int64_t koff = 0;
        uint32_t tile_at = 0, sb_at = 0, small_at_ = 0, block_at = 0;
        for (int t = 0; t < ns; ++t) {
            const int64_t nt = seg_offsets[t + 1] - seg_offsets[t];
            SegInfo& g = segs[t];
            std::memset(&g, 0, sizeof(g));
            g.begin = seg_offsets[t]; g.end = seg_offsets[t + 1]; g.koff = koff;
            g.tile0 = g.tile1 = tile_at; g.samp0 = sb_at;
            g.rep = seg_copies(nt, false); g.pool0 = block_at; block_at += (uint32_t)n_cf * g.rep;
            if (small_ok && nt <= SMALL_MAX) {
                g.small = 1;
                small_list[small_at_++] = (uint32_t)t;
            } else {
                tile_at += (uint32_t)((nt + TW - 1) / TW); g.tile1 = tile_at;
                g.samp_cnt = sample_count((uint64_t)nt, cf_min, cf_max, false);
                const uint32_t nb = (g.samp_cnt + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
                for (uint32_t b = 0; b < nb; ++b) sblock_seg[sb_at + b] = (uint32_t)t;
                sb_at += nb;
            }
            for (int j = 0; j < n_cf; ++j) ktab[(size_t)t * n_cf + j] = (uint32_t)gravac_topk_count(nt, cf_list[j]);
            koff += ktab[(size_t)t * n_cf + commit];
        }
    }
    p.total_out = total_out;
    if (ev && hipEventRecord((hipEvent_t)ev->call_begin, stream) != hipSuccess) {
        if (slot) staging_release(slot, false);
        return GRAVAC_ERR_HIP;
    }
    if (slot) {
        bool copied;
        // the buffer as a kernel of the current device addresses it (none: only a copy can read it)
        void* dev = nullptr;
        if (hipHostGetDevicePointer(&dev, slot->mem, 0) != hipSuccess) { dev = nullptr; (void)hipGetLastError(); }
        if (dev) {
            const uint32_t n16 = (uint32_t)(table_bytes / 16);
            hipLaunchKernelGGL(table_copy_kernel, dim3((n16 + 255) / 256), dim3(256), 0, stream, (const uint4*)dev,
                               (uint4*)(ws + L.tables), n16);
            copied = hipGetLastError() == hipSuccess;
        } else {
            copied = hipMemcpyAsync(ws + L.tables, slot->mem, table_bytes, hipMemcpyHostToDevice, stream) == hipSuccess;
        }
        bool recorded = copied && hipEventRecord(slot->done, stream) == hipSuccess;
        // a copy that is queued but not followed by the slot's event: wait for it here, so that the slot is not
        // rewritten under it
        if (copied && !recorded) (void)hipStreamSynchronize(stream);
        staging_release(slot, recorded);
        if (!copied || !recorded) return GRAVAC_ERR_HIP;
    }

    const uint32_t tile_grid = (p.n_tiles + WAVES - 1) / WAVES;
    const uint32_t sub_grid = (p.n_tiles * SUB + WAVES - 1) / WAVES;
    const uint32_t light_grid = (p.n_tiles + LWAVES - 1) / LWAVES;
    const uint32_t scan_slices = (max_seg_tiles + SCAN_SLICE - 1) / SCAN_SLICE;

    const int ncf_form = n_cf <= 1 ? 0 : n_cf <= 2 ? 1 : n_cf <= 3 ? 2 : n_cf <= 4 ? 3 : 4;
    static_assert(MAXCF >= 4, "forms for 1, 2, 3, 4 and MAXCF CFs");
    static_assert(DENSE_ROUNDS == 4, "forms of the sampling kernel for 1, 2 and 4 groups per thread");
    // (a layerwise call takes SAMPLE_BLOCK samples per block; its small tensors are extra workgroups of this launch)
    const bool have_tiles = p.n_tiles != 0;  // (not if every tensor of a layerwise call is small)
    if (have_tiles && !fixed) {              // (the threshold sparsifier uses nothing of what this kernel samples or clears)
        void (*const sample_forms[3])(Params) = {sample_kernel<1>, sample_kernel<2>, sample_kernel<4>};
        hipLaunchKernelGGL(sample_forms[sample_rounds == 1 ? 0 : sample_rounds == 2 ? 1 : 2], dim3(p.n_sample_blocks), dim3(256),
                           0, stream, p);
    }
    // a layerwise call's small tensors are done by their workgroups of this launch; few segments (none of them small):
    // their sample histograms are added up by SGRP workgroups each; many: by one each
    if (n_small)
        hipLaunchKernelGGL((threshold_kernel<1, true>), dim3(ns, 1), dim3(1024), 0, stream, p);
    else if (ns <= 32 && p.bounds_from == BOUNDS_SAMPLED)
    {
        if (p.n_sample_blocks > 64u * (uint32_t)ns)
            hipLaunchKernelGGL((threshold_kernel<SGRP, false, 4>), dim3(ns, SGRP), dim3(4096 / SGRP), 0, stream, p);
        else
            hipLaunchKernelGGL((threshold_kernel<SGRP, false, 2>), dim3(ns, SGRP), dim3(2048 / SGRP), 0, stream, p);
    }
    else
        hipLaunchKernelGGL((threshold_kernel<1, false>), dim3(ns, 1), dim3(1024), 0, stream, p);
    {
        // the Top-k pass exists in forms for 1, 2, 3, 4 and MAXCF CFs (its loops over the CFs are unrolled)
        void (*const ef_forms[5])(Params) = {stream_kernel<SM_EF, false, 1>, stream_kernel<SM_EF, false, 2>,
                                             stream_kernel<SM_EF, false, 3>, stream_kernel<SM_EF, false, 4>,
                                             stream_kernel<SM_EF, false, MAXCF>};
        void (*kern)(Params) = single ? stream_kernel<SM_SINGLE, false, 1>   // (a second-level call has one CF)
                                      : (random ? stream_kernel<SM_EF, true, MAXCF> : ef_forms[ncf_form]);
        if (!have_tiles) {
            if (ev) { (void)hipEventRecord((hipEvent_t)ev->pass_begin, stream); (void)hipEventRecord((hipEvent_t)ev->pass_end, stream); }
        } else if (ev)  // the kernel's own begin and end time stamps
            hipExtLaunchKernelGGL(kern, dim3(sub_grid), dim3(WG), 0, stream, (hipEvent_t)ev->pass_begin,
                                  (hipEvent_t)ev->pass_end, 0, p);
        else
            hipLaunchKernelGGL(kern, dim3(sub_grid), dim3(WG), 0, stream, p);
    }
    if (have_tiles && !fixed) {
    hipLaunchKernelGGL(locate_kernel, dim3((uint32_t)(ns * n_cf)), dim3(256), 0, stream, p);
    // exact routes, taken only by segments whose bracket failed (the kernels return at once otherwise)
    hipLaunchKernelGGL(coarse_kernel, dim3(tile_grid < XGRID ? tile_grid : XGRID), dim3(WG), 0, stream, p);
    if (random)
        hipLaunchKernelGGL((stream_kernel<SM_EXACT, true, MAXCF>), dim3(sub_grid < XGRID ? sub_grid : XGRID), dim3(WG), 0, stream, p);
    else
        hipLaunchKernelGGL((stream_kernel<SM_EXACT, false, MAXCF>), dim3(sub_grid < XGRID ? sub_grid : XGRID), dim3(WG), 0, stream, p);
    }
    if (have_tiles) {
    // the refine kernel loops over the CFs: forms for 1, 2, 3, 4 and MAXCF CFs
    // (... and with or without the early loads of the lists' heads: with them if the tiles' wavefronts are all resident
    // at once, six per SIMD on 1024 SIMDs)
    void (*const refine_forms[2][5])(Params) = {
        {refine_kernel<1, false>, refine_kernel<2, false>, refine_kernel<3, false>, refine_kernel<4, false>, refine_kernel<MAXCF, false>},
        {refine_kernel<1, true>, refine_kernel<2, true>, refine_kernel<3, true>, refine_kernel<4, true>, refine_kernel<MAXCF, true>}};
    const int heads = (!random && p.n_tiles <= 6144u) ? 1 : 0;
    hipLaunchKernelGGL(refine_forms[heads][ncf_form], dim3(light_grid), dim3(LWG), 0, stream, p);
    hipLaunchKernelGGL(scan_kernel, dim3(ns, scan_slices + n_cf), dim3(SCAN_T), 0, stream, p, scan_slices);
    {
        // (the plain call's form with the early loads of the lists' heads if the tiles' wavefronts are all resident at once)
        void (*emit)(Params) = (p.random || p.single) ? emit_kernel<true, false>
                                                      : (p.n_tiles <= 6144u ? emit_kernel<false, true> : emit_kernel<false, false>);
        hipLaunchKernelGGL(emit, dim3(light_grid), dim3(LWG), 0, stream, p);
    }
    }
    if (ev) (void)hipEventRecord((hipEvent_t)ev->call_end, stream);
    if (hipGetLastError() != hipSuccess) return GRAVAC_ERR_HIP;
    return GRAVAC_OK;
}

int gravac_compress(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                    const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val, int64_t out_capacity,
                    int64_t* out_count, double* out_stats, void* workspace, size_t workspace_bytes, unsigned flags,
                    void* stream_v)
{
    if (!residual) return GRAVAC_ERR_INVALID_ARG;
    return compress_impl(grad, residual, n, cf_list, n_cf, commit, seg_offsets, n_seg, out_idx, out_val, out_capacity,
                         out_count, out_stats, workspace, workspace_bytes, flags, (hipStream_t)stream_v, nullptr, nullptr, 0,
                         nullptr, nullptr);
}

int gravac_compress_profiled(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                             const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val,
                             int64_t out_capacity, int64_t* out_count, double* out_stats, void* workspace,
                             size_t workspace_bytes, unsigned flags, void* stream_v, const gravac_profile_events* events)
{
    if (!residual || !events) return GRAVAC_ERR_INVALID_ARG;
    return compress_impl(grad, residual, n, cf_list, n_cf, commit, seg_offsets, n_seg, out_idx, out_val, out_capacity,
                         out_count, out_stats, workspace, workspace_bytes, flags, (hipStream_t)stream_v, nullptr, nullptr, 0,
                         nullptr, events);
}

int gravac_randomk_compress(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                            uint64_t seed, const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val,
                            int64_t out_capacity, int64_t* out_count, double* out_stats, void* workspace,
                            size_t workspace_bytes, unsigned flags, void* stream_v)
{
    if (!residual) return GRAVAC_ERR_INVALID_ARG;
    return compress_impl(grad, residual, n, cf_list, n_cf, commit, seg_offsets, n_seg, out_idx, out_val, out_capacity,
                         out_count, out_stats, workspace, workspace_bytes, flags, (hipStream_t)stream_v, nullptr, nullptr, 0,
                         &seed, nullptr);
}

int gravac_threshold_compress(const float* grad, float* residual, int64_t n, float tau, int32_t* out_idx, float* out_val,
                              int64_t out_capacity, int64_t* out_count, double* out_stats, void* workspace,
                              size_t workspace_bytes, void* stream_v)
{
    if (!residual) return GRAVAC_ERR_INVALID_ARG;
    const double one = 1.0;
    return compress_impl(grad, residual, n, &one, 1, 0, nullptr, 0, out_idx, out_val, out_capacity, out_count, out_stats,
                         workspace, workspace_bytes, 0, (hipStream_t)stream_v, nullptr, nullptr, 0, nullptr, nullptr, &tau);
}

int gravac_recompress(const int32_t* idx1, const float* val1, int64_t k1, double cf_rel, const int64_t* seg_counts,
                      int n_seg, float* residual, int64_t n, int32_t* out_idx, float* out_val, int64_t out_capacity,
                      int64_t* out_count, double* out_stats, void* workspace, size_t workspace_bytes, unsigned flags,
                      void* stream_v)
{
    if (!idx1 || !val1 || k1 <= 0 || n_seg < 0 || (n_seg > 0 && !seg_counts)) return GRAVAC_ERR_INVALID_ARG;
    if (residual && (n <= 0 || n > 2147483647LL)) return GRAVAC_ERR_INVALID_ARG;
    std::vector<int64_t> off;
    if (n_seg > 0) {
        off.resize((size_t)n_seg + 1);
        off[0] = 0;
        for (int t = 0; t < n_seg; ++t) {
            if (seg_counts[t] <= 0 || seg_counts[t] > k1) return GRAVAC_ERR_INVALID_ARG;
            off[t + 1] = off[t] + seg_counts[t];
        }
        if (off[n_seg] != k1) return GRAVAC_ERR_INVALID_ARG;
    }
    return compress_impl(val1, nullptr, k1, &cf_rel, 1, 0, n_seg > 0 ? off.data() : nullptr, n_seg, out_idx, out_val,
                         out_capacity, out_count, out_stats, workspace, workspace_bytes, flags, (hipStream_t)stream_v,
                         idx1, residual, n, nullptr, nullptr);
}

int gravac_commit(const int32_t* idx, int64_t count, float* residual, int64_t n, void* stream_v)
{
    if (!residual || count < 0 || n <= 0 || n > 2147483647LL || (count > 0 && !idx)) return GRAVAC_ERR_INVALID_ARG;
    if (count == 0) return GRAVAC_OK;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(commit_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream_v, idx, count, residual, n);
    if (hipGetLastError() != hipSuccess) return GRAVAC_ERR_HIP;
    return GRAVAC_OK;
}

int gravac_decompress_workspace_bytes(int W, int64_t n, size_t* bytes_out)
{
    if (!bytes_out || W < 1 || n <= 0 || n > 2147483647LL) return GRAVAC_ERR_INVALID_ARG;
    const int64_t ntile = (n + DTILE - 1) / DTILE;
    const int wn = W < DMAXW ? W : DMAXW;
    *bytes_out = align_up(sizeof(uint32_t) * (size_t)wn * (size_t)(ntile + 1), 256);
    return GRAVAC_OK;
}

// bounds: device memory for the tile boundaries of up to DMAXW messages (the caller's workspace or the library's static
// scratch, already checked for size), or null for the search path.
static int decompress_impl(const int32_t* idx, const float* val, const int64_t* counts, int W, int64_t n, float* dense_out,
                           float alpha, uint32_t* bounds, void* stream_v)
{
    hipStream_t stream = (hipStream_t)stream_v;
    if (!counts || !dense_out || W < 1 || n <= 0 || n > 2147483647LL) return GRAVAC_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int w = 0; w < W; ++w) {
        if (counts[w] < 0) return GRAVAC_ERR_INVALID_ARG;
        total += counts[w];
    }
    if (total > 0 && (!idx || !val)) return GRAVAC_ERR_INVALID_ARG;
    if (total == 0) return GRAVAC_OK;
    const int64_t ntile = (n + DTILE - 1) / DTILE;
    const uint32_t grid = (uint32_t)(ntile < 1024 ? ntile : 1024);  // 4 workgroups (4 x 32 KiB LDS) on each of 256 CUs
    int64_t at = 0;
    for (int w0 = 0; w0 < W; w0 += DMAXW) {
        const int wn = (W - w0 < DMAXW) ? W - w0 : DMAXW;
        WorkerOffsets wo;
        int64_t group = 0, longest = 0;
        for (int w = 0; w < wn; ++w) {
            wo.at[w] = at + group;
            group += counts[w0 + w];
            if (counts[w0 + w] > longest) longest = counts[w0 + w];
        }
        for (int w = wn; w <= DMAXW; ++w) wo.at[w] = at + group;
        at += group;
        if (group == 0) continue;
        if (bounds) {
            // tile boundaries of the group's messages first (the workspace is reused from group to group: stream order)
            const uint32_t pair_blocks = (uint32_t)((longest + 255) / 256);
            hipLaunchKernelGGL(bounds_kernel, dim3(pair_blocks, (uint32_t)wn), dim3(256), 0, stream, idx, wo, ntile,
                               bounds);
            hipLaunchKernelGGL(decompress_ws_kernel, dim3(grid), dim3(256), 0, stream, idx, val, wo, wn, n, dense_out,
                               (const uint32_t*)bounds, alpha);
        } else {
            hipLaunchKernelGGL(decompress_kernel, dim3(grid), dim3(256), 0, stream, idx, val, wo, wn, n, dense_out, alpha);
        }
    }
    if (hipGetLastError() != hipSuccess) return GRAVAC_ERR_HIP;
    return GRAVAC_OK;
}


int gravac_decompress_accumulate(const int32_t* idx, const float* val, const int64_t* counts, int W, int64_t n,
                                 float* dense_out, void* workspace, size_t workspace_bytes, void* stream_v)
{
    if (!counts || !dense_out || W < 1 || n <= 0 || n > 2147483647LL) return GRAVAC_ERR_INVALID_ARG;
    if (workspace) {
        size_t need = 0;
        if (gravac_decompress_workspace_bytes(W, n, &need) != GRAVAC_OK) return GRAVAC_ERR_INVALID_ARG;
        if (((uintptr_t)workspace & 255) || workspace_bytes < need) return GRAVAC_ERR_WORKSPACE;
    }
    return decompress_impl(idx, val, counts, W, n, dense_out, 1.0f, (uint32_t*)workspace, stream_v);
}

int gravac_decompress_update(const int32_t* idx, const float* val, const int64_t* counts, int W, int64_t n, float alpha,
                             float* params, void* workspace, size_t workspace_bytes, void* stream_v)
{
    if (!counts || !params || W < 1 || n <= 0 || n > 2147483647LL) return GRAVAC_ERR_INVALID_ARG;
    if (workspace) {
        size_t need = 0;
        if (gravac_decompress_workspace_bytes(W, n, &need) != GRAVAC_OK) return GRAVAC_ERR_INVALID_ARG;
        if (((uintptr_t)workspace & 255) || workspace_bytes < need) return GRAVAC_ERR_WORKSPACE;
    }
    return decompress_impl(idx, val, counts, W, n, params, alpha, (uint32_t*)workspace, stream_v);
}

int gravac_decompress_accumulate_static(const int32_t* idx, const float* val, const int64_t* counts, int W, int64_t n,
                                        float* dense_out, void* stream_v)
{
    if (!counts || !dense_out || W < 1 || n <= 0 || n > 2147483647LL) return GRAVAC_ERR_INVALID_ARG;
    size_t need = 0;
    if (gravac_decompress_workspace_bytes(W, n, &need) != GRAVAC_OK) return GRAVAC_ERR_INVALID_ARG;
    if (need > (size_t)GRAVAC_STATIC_SCRATCH_BYTES) return GRAVAC_ERR_STATIC_LIMIT;
    uint32_t* bounds = nullptr;
    if (const int rc = static_scratch(&bounds)) return rc;
    return decompress_impl(idx, val, counts, W, n, dense_out, 1.0f, bounds, stream_v);
}

int gravac_read_status(const void* workspace, void* stream_v, int32_t* out8)
{
    if (!workspace || !out8) return GRAVAC_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_v;
    if (hipStreamSynchronize(stream) != hipSuccess) return GRAVAC_ERR_HIP;
    Status s;
    if (hipMemcpy(&s, workspace, sizeof(Status), hipMemcpyDeviceToHost) != hipSuccess) return GRAVAC_ERR_HIP;
    out8[0] = s.any_fail; out8[1] = s.n_fail; out8[2] = s.error; out8[3] = s.n_seg; out8[4] = s.n_narrow;
    out8[5] = out8[6] = out8[7] = 0;
    return GRAVAC_OK;
}

const char* gravac_strerror(int code)
{
    switch (code) {
        case GRAVAC_OK: return "ok";
        case GRAVAC_ERR_INVALID_ARG: return "invalid argument";
        case GRAVAC_ERR_CAPACITY: return "output capacity too small";
        case GRAVAC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case GRAVAC_ERR_HIP: return "HIP runtime error";
        case GRAVAC_ERR_STATIC_LIMIT: return "W and n exceed what the library's static scratch holds";
        case GRAVAC_ERR_CAPTURE: return "call cannot be recorded into a HIP graph (layerwise or profiled call on a capturing stream)";
        default: return "unknown error code";
    }
}

}  // extern "C"
