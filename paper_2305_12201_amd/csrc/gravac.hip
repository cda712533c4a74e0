// gravac.hip - Top-k + error-feedback gradient compression for MI355X (gfx950).
//
// Implements the C ABI of include/gravac.h.  The path follows GraVAC (arxiv 2305.12201):
// error feedback (Sec. III-B), Top-k sparsification at a compression factor (Sec. II-C),
// residual update (Alg. 1), compression gain for several candidate CFs (Sec. III-B
// equation, Alg. 1 gain steps), layerwise mode and decompression (Sec. III-A).
//
// Design in one paragraph.  Keys are the binary32 bit patterns of |acc|, so magnitude order is
// unsigned-integer order.  A small strided sample of acc gives, per candidate CF, a lower bound
// `lo` on the k-th largest key (with a statistical safety margin) and a shift `s`.  ONE streaming
// pass then reads grad and residual, writes acc back as the provisional residual, sums acc^2 and
// diverts every element with key >= lo (a few k of them) into an index-ordered per-tile
// candidate list, histogramming those candidates by (key - lo) >> s.  Everything after that
// works on the candidate lists only: locate the histogram bin that holds the k-th largest,
// resolve it to the exact key, count per tile, and emit the message in ascending index order
// while zeroing the selected residual slots.  If the sampled bound turns out wrong the segment is
// redone by a route that cannot fail: a bin too coarse and too full to resolve is binned again inside
// itself; a k-th largest above the bracket is found from a 2048-bin histogram of the candidates'
// top key bits; with fewer than k candidates that histogram is built over all elements and the
// candidates are collected again.  Results are identical on every route; only the number of
// passes over memory differs.
//
// Units of work.  A tile is TW consecutive elements; the streaming pass gives each of its SUB
// sub-tiles to one 64-lane wavefront, which owns that sub-tile's slots of the candidate arrays, so
// ordered compaction needs no communication between wavefronts and no list can overflow.  No kernel
// waits on another workgroup: cross-tile results (histograms, output offsets) are combined at kernel
// boundaries.  Global atomics complete at a rate of roughly one per cache line per 10 ns on this part,
// so the candidate histogram and the gather lists exist in REP copies (picked from the sub-tile,
// tile or workgroup number) and nothing else uses global atomics.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <vector>

#include "gravac.h"

namespace {

#ifndef GV_TW
#define GV_TW 8192
#endif
constexpr int TW = GV_TW;           // elements per tile (unit of the candidate-list kernels)
#ifndef GV_SUB
#define GV_SUB 8
#endif
constexpr int SUB = GV_SUB;         // sub-tiles per tile: the streaming pass gives one wavefront a sub-tile
constexpr int TS = TW / SUB;        // elements per sub-tile
constexpr int WG = 256;             // threads per workgroup of the tile kernels
constexpr int WAVES = WG / 64;
#ifndef GV_LWG
#define GV_LWG 256
#endif
constexpr int LWG = GV_LWG;         // threads per workgroup of the candidate-list kernels (refine, count, emit)
constexpr int LWAVES = LWG / 64;
constexpr int VCHUNK = 256;          // dense tiles: slots of one sub-tile list a wavefront takes per load, four per lane
constexpr int VLISTS = 4;            // ... from this many of the tile's lists at a time (registers)
constexpr uint32_t DENSE_TILE = TW / 4;  // a tile with at least this many candidates is walked that way
static_assert(TS % VCHUNK == 0, "a sub-tile list is a whole number of such chunks");
constexpr int ROW = 256;            // elements one wavefront touches per load (64 lanes x float4)
#ifndef GV_ROWS
#define GV_ROWS 4                   // rows a wavefront keeps in flight
#endif
#ifndef GV_NT
#define GV_NT 1                     // non-temporal hints on the streaming loads and stores
#endif
#ifndef GV_XGRID
#define GV_XGRID 1024
#endif
constexpr uint32_t XGRID = GV_XGRID;  // workgroups of the two exact-route kernels (they loop over the tiles)
constexpr int REP = 8;              // copies of the candidate histogram and of the gather lists
constexpr int NBIN = 2048;          // bins of the candidate / refine / coarse histograms
constexpr uint32_t OVF = NBIN - 1;  // last bin of the candidate histogram: everything above the bracket
constexpr int SBIN = 4096;          // bins of the sample histogram: 2^17 keys each (64 per octave, 1.1 % in magnitude)
constexpr uint32_t SSHIFT = 17;     // from |x| = 2^-48 up to 2^16; smaller magnitudes share bin 0, larger ones the last bin
constexpr uint32_t SKEY0 = 79u << 23;
static_assert((uint64_t)SKEY0 + ((uint64_t)SBIN << SSHIFT) <= 0x7F800000ull, "the window lies inside the finite keys");
constexpr int SAMPLE_BLOCK = 1024;  // samples per workgroup of the sampling kernel
constexpr int SAMPLE_MAX = 65536;   // samples per segment at most (unless the segment is read whole)
constexpr int SAMPLE_MAX_FLAT = 524288;  // flat mode, a large k: see sample_count
constexpr int DENSE_ROUNDS = 4;          // ... whose sample blocks are up to DENSE_ROUNDS * SAMPLE_BLOCK samples each
constexpr int DENSE_BLOCKS = 128;        // ... so that there are at most this many of them
constexpr int LCAP = 4096;          // keys a gather list can hold
constexpr int MAXCF = GRAVAC_MAX_CF;
constexpr uint32_t REUSE_MAX_K = 1u << 21;  // a CF that selects more entries than this is sampled even when thresholds are reused:
                                            // the bracket a sample gives holds fewer entries than 0.25 k below the old threshold
constexpr double ZMARGIN = 5.0;     // safety margin of the sampled rank, in standard deviations
constexpr uint32_t NONE = 0xFFFFFFFFu;

enum : uint32_t { MODE_RESOLVED = 0, MODE_GATHER = 1, MODE_HIST = 2, MODE_FAIL = 3 };
// SegState::fail, the heaviest kind over the segment's CFs wins:
//   FAIL_NARROW  the bin that holds the k-th largest is known but too coarse and too full to resolve: only the
//                CFs concerned are binned again, inside that bin (no other pass);
//   FAIL_LIGHT   the k-th largest lies above the histogram's bracket: the candidates hold it, all CFs of the
//                segment are binned again from a coarse histogram of the candidates;
//   FAIL_FULL    fewer than k candidates: acc is read again.
enum : uint32_t { FAIL_NONE = 0, FAIL_NARROW = 1, FAIL_LIGHT = 2, FAIL_FULL = 3 };

// Selection state of one (segment, CF).
struct CfState {
    uint32_t k;         // entries to select
    uint32_t lo;        // candidates for this CF have key >= lo
    uint32_t s;         // candidate-histogram bin = min((key - lo) >> s, OVF)
    uint32_t mode;      // MODE_*
    uint32_t base;      // first key of the bin that holds the k-th largest
    uint32_t open;      // 1 if that bin is the open-ended last bin
    uint32_t above;     // number of keys above that bin
    uint32_t c;         // number of keys in that bin
    uint32_t tau;       // key of the k-th largest (valid once resolved)
    uint32_t need;      // how many keys equal to tau are selected (lowest indices first)
    uint32_t cnt_gt;    // number of keys greater than tau
    uint32_t redo;      // 1 if this CF is binned again on the narrow route (set by the locate step)
    uint32_t lo2, s2;   // ... with these bounds: the located bin, cut into 1024 parts
    uint32_t pad[2];
};
static_assert(sizeof(CfState) == 64, "CfState layout");

struct SegState {
    uint32_t lo_min;  // smallest lo over the CFs: the candidate threshold of the segment
    uint32_t fail;    // FAIL_*: whether the bound failed and the segment takes the exact route, and which form of it
    uint32_t pz;      // the streaming pass has stored +0 instead of acc for keys >= pz: the upper end of the committed
                      // CF's bracket, above which an entry is selected unless the bound fails (NONE: nothing zeroed)
    uint32_t pad;
};

struct Status {
    int any_fail;
    int n_fail;
    int error;
    int n_seg;
    uint32_t sig_lo, sig_hi;  // signature (shape, CFs, segment table) of the last call that completed on this workspace
    int n_light;              // segments of n_fail whose exact route only re-binned the candidates
    int pad;
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
    uint32_t pad[6];
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
    uint32_t rk_s0, rk_s1;   // its two 31-bit keys (from the seed)
    int64_t n;
    int n_seg;  // >= 1
    int n_cf;
    int commit;
    unsigned flags;
    uint32_t sig_lo, sig_hi;  // signature of this call
    int64_t total_out;        // pairs the call emits
    uint32_t n_tiles;
    uint32_t n_sample_blocks;
    uint32_t have_sample;          // 1 if the sampling kernel has run for this call
    // layerwise tables in the workspace (unused when n_seg == 1)
    const SegInfo* segs;           // [n_seg] built on the host
    const uint32_t* ktab;          // [n_seg][n_cf] built on the host
    const uint32_t* sblock_seg;    // [n_sample_blocks] segment of every sample block, built on the host
    uint32_t* tseg;                // [n_tiles] segment of every tile, filled by threshold_kernel
    // the same for one flat tensor
    uint32_t flat_k[MAXCF];
    uint32_t flat_samples;
    // workspace
    Status* status;
    CfState* st;         // [n_seg][n_cf]
    SegState* seg;       // [n_seg]
    uint32_t* hist1;     // [n_seg][n_cf][REP][NBIN] candidate histogram, REP copies
    uint32_t* ovfc;      // [n_seg][n_cf][64][32] counts above the bracket (the histogram's last bin), spread over
                         // 64 cache lines; word 0 of each line is used
    uint32_t* hist2;     // [n_seg][n_cf][NBIN] refine histogram
    uint32_t* coarse;    // [n_seg][NBIN] histogram of key >> 20 (exact route)
    uint32_t* list;      // [n_seg][n_cf][REP][LCAP] gather lists, REP copies
    uint32_t* list_cnt;  // [n_seg][n_cf][REP][32] fill counts of the gather lists, one cache line each
    uint32_t* samp_hist; // [n_sample_blocks][SBIN / 2] sample histograms, two 16-bit counts per word
    uint32_t* cand_cnt;  // [n_tiles][SUB] candidates of every sub-tile
    uint32_t* tg;        // [n_tiles] candidates above tau(commit) in this tile
    uint32_t* te;        // [n_tiles] candidates equal to tau(commit) in this tile
    uint32_t* toff;      // [n_tiles] offset of the tile's output inside its segment's message
    uint32_t* ttake;     // [n_tiles] how many of the tile's candidates equal to tau(commit) are selected
    double* ssd;         // [n_tiles][SUB] sum of acc^2 of every sub-tile
    double* ssd_t;       // [n_tiles] sum of acc^2 of the tile
    double* sss;         // [n_tiles][n_cf] sum of acc^2 over keys > tau_j
    int32_t* cand_idx;   // [n_tiles][SUB][TS] sub-tile j of tile u owns the slots from (u*SUB + j)*TS
    float* cand_val;     // [n_tiles][SUB][TS]
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

__device__ __forceinline__ uint32_t key_of(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

// Bin of the sample histogram a key falls into, and the keys a bin spans.
__device__ __forceinline__ uint32_t sample_bin(uint32_t key)
{
    if (key < SKEY0) return 0u;
    const uint32_t b = (key - SKEY0) >> SSHIFT;
    return b < (uint32_t)SBIN - 1u ? b : (uint32_t)SBIN - 1u;
}
__device__ __forceinline__ uint32_t sample_bin_first(uint32_t b) { return b == 0u ? 0u : SKEY0 + (b << SSHIFT); }
__device__ __forceinline__ uint64_t sample_bin_end(uint32_t b)
{
    return b == (uint32_t)SBIN - 1u ? 2147483648ull : (uint64_t)SKEY0 + ((uint64_t)(b + 1u) << SSHIFT);
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

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// inclusive prefix sum over the lanes of a wavefront
__device__ __forceinline__ uint32_t wave_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t x = __shfl_up(v, o, 64);
        if (lane >= o) v += x;
    }
    return v;
}

__device__ __forceinline__ uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// The candidates of a tile are the concatenation of its SUB sub-tile lists.
struct TileCands {
    uint32_t start[SUB + 1];  // start[j] = candidates in sub-tiles before j; start[SUB] = all
    __device__ __forceinline__ uint32_t total() const { return start[SUB]; }
    __device__ __forceinline__ uint32_t longest() const  // candidates of the fullest sub-tile
    {
        uint32_t m = 0;
#pragma unroll
        for (int j = 0; j < SUB; ++j) m = max(m, start[j + 1] - start[j]);
        return m;
    }
    // slot (relative to the tile's first slot) of the tile's i-th candidate
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

__device__ __forceinline__ TileCands tile_cands(const Params& p, uint32_t u)
{
    TileCands c;
    c.start[0] = 0;
#pragma unroll
    for (int j = 0; j < SUB; ++j) c.start[j + 1] = c.start[j] + p.cand_cnt[(size_t)u * SUB + j];
    return c;
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
// K0a: sample acc = residual + grad at stratified positions; each workgroup histograms its samples in
// LDS (SBIN bins of 2^17 keys, see sample_bin) and stores the counts as 16-bit numbers
// ---------------------------------------------------------------------------------------------
template <int R>  // R groups per thread: a workgroup histograms R * SAMPLE_BLOCK samples
__global__ __launch_bounds__(256) void sample_kernel(Params p)
{
    __shared__ uint32_t h[SBIN];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const int t = is_flat(p) ? 0 : (int)p.sblock_seg[b];
    const uint32_t lb = b - (is_flat(p) ? 0u : p.segs[t].samp0);
    const uint32_t S = is_flat(p) ? p.flat_samples : p.segs[t].samp_cnt;
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
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t g = (lb * R + r) * (SAMPLE_BLOCK / 4) + tid;  // group
        gpos[r] = 4ull * g;                                          // the whole segment is read: elements 4g .. 4g+3
        if ((uint64_t)S != nt) {
            // four neighbouring threads share one stratum and one run of 16 elements in it that starts at a multiple
            // of 16 in the flat buffer (a 64-byte line if the buffer is aligned to that)
            const uint32_t g16 = g >> 2;
            const uint64_t G = S / 16, a = ((uint64_t)g16 * nt) / G, e = ((uint64_t)(g16 + 1) * nt) / G;  // e - a >= 32
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
#pragma unroll
    for (int m = 0; m < 8; ++m) wp[m] = h[16 * tid + 2 * m] | (h[16 * tid + 2 * m + 1] << 16);
    uint4* dst = (uint4*)(p.samp_hist + (size_t)b * (SBIN / 2) + 8 * tid);
    dst[0] = w[0];
    dst[1] = w[1];
}

// ---------------------------------------------------------------------------------------------
// K0b: per segment, add up the sample histograms and turn them into (lo, s) per CF; clear the
// segment's histograms and gather-list counts
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void threshold_kernel(Params p)
{
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t rank_lo[MAXCF], rank_hi[MAXCF], bin_lo[MAXCF], bin_hi[MAXCF];
    const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    const uint32_t S = is_flat(p) ? p.flat_samples : p.segs[t].samp_cnt;
    const uint32_t sb0 = is_flat(p) ? 0u : p.segs[t].samp0;
    const uint32_t nb = is_flat(p) ? p.n_sample_blocks : (S + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
    if (!is_flat(p))
        for (uint32_t u = seg_tile0(p, t) + tid; u < seg_tile1(p, t); u += 1024) p.tseg[u] = (uint32_t)t;
    const uint64_t nt = (uint64_t)(seg_end(p, t) - seg_begin(p, t));
    const bool whole = ((uint64_t)S == nt);
    // reuse: take the previous call's thresholds as bounds, if that call had this call's signature;
    // without a usable prediction (and without samples) every segment takes the exact route
    const bool want_reuse = (p.flags & GRAVAC_FLAG_REUSE_THRESHOLDS) != 0;
    const bool reuse = want_reuse && p.status->sig_lo == p.sig_lo && p.status->sig_hi == p.sig_hi;
    // (a call that reuses thresholds samples as well if one of its CFs selects more than REUSE_MAX_K entries: such a CF
    // takes its bounds from the sample, and so does every CF if the workspace turns out to hold no matching call)
    const bool forced = (p.flags & GRAVAC_FLAG_FORCE_FALLBACK) != 0 || (want_reuse && !reuse && !p.have_sample);
    const bool sampled = !forced && !p.random && p.have_sample != 0;

    // reuse: the previous call's candidate histogram says where its count from the top reached about 1.25 k;
    // that key becomes this call's lower bound (wavefront j looks at CF j, before the histogram is cleared)
    __shared__ uint32_t pred_lo[MAXCF];
    __shared__ uint32_t team_scratch[4][8];
    if (reuse) {
        // four teams of four wavefronts, team g takes CF g and CF g + 4
        const int team = tid >> 8, q = tid & 255;
        for (int r = 0; r < (p.n_cf + 3) / 4; ++r) {
            const int j = r * 4 + team;
            const int jj = j < p.n_cf ? j : 0;  // idle teams repeat CF 0 (they must reach the barriers)
            const CfState* old = &p.st[(size_t)t * p.n_cf + jj];
            const uint32_t k = seg_k(p, t, jj), lo_prev = old->lo, s_prev = old->s > 31u ? 31u : old->s;
            uint32_t b, ab, cn;
            team_locate_bin(p.hist1 + ((size_t)t * p.n_cf + jj) * REP * NBIN, REP, p.ovfc + ((size_t)t * p.n_cf + jj) * 64 * 32,
                            k + k / 4 + 64, q, team_scratch[team], [] { __syncthreads(); }, b, ab, cn);
            uint32_t lo;
            // fewer candidates than that: go lower; a tensor of at most LCAP elements takes all its elements for one
            // call (whatever bin then holds its k-th largest can be gathered), after which its histogram reaches the level
            if (b == NONE) lo = (nt > (uint64_t)LCAP && lo_prev > (1u << 19)) ? lo_prev - (1u << 19) : 0u;
            else {
                const uint64_t x = (uint64_t)lo_prev + ((uint64_t)b << s_prev);
                lo = x > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)x;
            }
            if (q == 0 && j < p.n_cf) pred_lo[j] = lo;
        }
    }
    __syncthreads();
    for (int i = tid; i < p.n_cf * REP * NBIN; i += 1024) p.hist1[(size_t)t * p.n_cf * REP * NBIN + i] = 0;
    for (int i = tid; i < NBIN; i += 1024) p.coarse[(size_t)t * NBIN + i] = 0;
    for (int i = tid; i < p.n_cf * 64; i += 1024) p.ovfc[((size_t)t * p.n_cf * 64 + i) * 32] = 0;
    for (int i = tid; i < p.n_cf * REP * 32; i += 1024) p.list_cnt[(size_t)t * p.n_cf * REP * 32 + i] = 0;
    if (t == 0 && tid == 0) {
        p.status->any_fail = 0; p.status->n_fail = 0; p.status->error = 0; p.status->n_seg = p.n_seg;
        p.status->n_light = 0;
    }
    if (tid < p.n_cf) {
        const uint32_t k = seg_k(p, t, tid);
        uint32_t r_lo, r_hi;
        if (whole) {
            r_lo = r_hi = k;
        } else {
            // expected number of sampled keys among the k largest, widened by ZMARGIN standard deviations
            const double m = (double)k * (double)S / (double)nt, sd = sqrt(m);
            const double a = ceil(m + ZMARGIN * sd + 2.0), b = floor(m - ZMARGIN * sd - 2.0);
            r_lo = (a >= 4.0e9) ? NONE : (uint32_t)a;
            r_hi = (b < 1.0) ? 1u : (uint32_t)b;
        }
        rank_lo[tid] = r_lo; rank_hi[tid] = r_hi;
        bin_lo[tid] = 0;            // fewer than r_lo samples (or none at all): every key is a candidate
        bin_hi[tid] = SBIN - 1;
    }

    // thread i owns bins 4i .. 4i+3: two words of every block's histogram
    uint32_t h0 = 0, h1 = 0, h2 = 0, h3 = 0;
    if (sampled) {
        const uint2* src = (const uint2*)(p.samp_hist + (size_t)sb0 * (SBIN / 2)) + tid;
        for (uint32_t b0 = 0; b0 < nb; b0 += 32) {
            uint2 w[32];
#pragma unroll
            for (int q = 0; q < 32; ++q) w[q] = (b0 + q < nb) ? src[(size_t)(b0 + q) * (SBIN / 4)] : make_uint2(0u, 0u);
#pragma unroll
            for (int q = 0; q < 32; ++q) {
                h0 += w[q].x & 0xFFFFu; h1 += w[q].x >> 16;
                h2 += w[q].y & 0xFFFFu; h3 += w[q].y >> 16;
            }
        }
    }
    const uint32_t mine = h0 + h1 + h2 + h3;
    const uint32_t incl = wave_scan(mine);
    if (lane == 63) wtot[wib] = incl;
    __syncthreads();
    uint32_t total = 0, before = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const uint32_t x = wtot[w];
        total += x;
        if (w < wib) before += x;
    }
    const uint32_t above0 = total - (before + incl);  // samples in bins above this thread's four
    const uint32_t hh[4] = {h0, h1, h2, h3};
    for (int j = 0; j < p.n_cf; ++j) {
        const uint32_t r_lo = rank_lo[j], r_hi = rank_hi[j];
        uint32_t above = above0;
#pragma unroll
        for (int q = 3; q >= 0; --q) {
            const uint32_t c = hh[q];
            if (above < r_lo && above + c >= r_lo) bin_lo[j] = 4 * tid + q;
            if (above < r_hi && above + c >= r_hi) bin_hi[j] = 4 * tid + q;
            above += c;
        }
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t lo_min = NONE, pz = NONE;
        for (int j = 0; j < p.n_cf; ++j) {
            uint32_t lo = sample_bin_first(bin_lo[j]);             // lower edge of the bin of the r_lo-th sample
            uint64_t hi = sample_bin_end(bin_hi[j]);               // upper edge of the bin of the r_hi-th sample
            if (reuse && !(sampled && seg_k(p, t, j) > REUSE_MAX_K)) {
                // from the key below which the previous call counted about 1.25 k candidates to 2^19 keys (about 4 % in
                // magnitude) above the previous threshold: tight, for a run in steady state; a threshold that moves
                // further than that costs one call through the exact route
                const uint32_t tau_prev = p.st[(size_t)t * p.n_cf + j].tau & 0x7FFFFFFFu;
                lo = pred_lo[j] < tau_prev ? pred_lo[j] : tau_prev;
                hi = (uint64_t)tau_prev + (1u << 19);

            }
            if (p.random) {
                // priorities are a keyed permutation of the 31-bit integers: the number of a tensor's nt indices
                // with priority >= x is as good as binomial (nt, 1 - x / 2^31), so the bounds follow from k alone:
                // x with k + ZMARGIN sqrt(k) + 2 expected above it, and x with k - ZMARGIN sqrt(k) - 2
                const double k = (double)seg_k(p, t, j), w = ZMARGIN * sqrt(k) + 2.0;
                const double q_lo = (k + w) / (double)nt, q_hi = (k - w) / (double)nt;
                lo = q_lo >= 1.0 ? 0u : (uint32_t)floor(2147483648.0 * (1.0 - q_lo));
                hi = q_hi <= 0.0 ? 2147483648ull : (uint64_t)ceil(2147483648.0 * (1.0 - q_hi));
            }
            uint32_t s = 0;
            while (((hi > lo ? hi - lo : 0) >> s) > (uint64_t)OVF) ++s;
            if (forced) { lo = NONE; s = 0; }
            CfState st;
            st.k = seg_k(p, t, j); st.lo = lo; st.s = s; st.mode = MODE_FAIL; st.base = 0; st.open = 0; st.above = 0;
            st.c = 0; st.tau = 0; st.need = 0; st.cnt_gt = 0;
            st.redo = 0; st.lo2 = 0; st.s2 = 0; st.pad[0] = st.pad[1] = 0;
            p.st[(size_t)t * p.n_cf + j] = st;
            lo_min = lo < lo_min ? lo : lo_min;
            if (j == p.commit && !forced && !p.single) {
                const uint64_t top = (uint64_t)lo + ((uint64_t)OVF << s);  // first key of the histogram's open last bin
                if (top <= 0x7FFFFFFFull) pz = (uint32_t)top;
            }
        }
        SegState ss;
        ss.lo_min = lo_min; ss.fail = 0; ss.pz = pz; ss.pad = 0;
        p.seg[t] = ss;
    }
}

// ---------------------------------------------------------------------------------------------
// K1: the streaming pass, one wave tile per wavefront.
//     EF = true: read grad and residual, write acc back, sum acc^2.
//     EF = false (exact route, failed segments only): read acc from residual; lo comes from the
//     coarse histogram.  Both collect the candidates of the tile in index order.
// ---------------------------------------------------------------------------------------------
struct TileCtx {
    uint32_t lo_min;
    uint32_t lo[MAXCF];
    uint32_t sh[MAXCF];
    uint32_t ovf[MAXCF];
    uint32_t* h1;   // this workgroup's copy of the candidate histograms of the tile's segment (CF stride REP*NBIN)
    int32_t* cidx;  // candidate slots of this tile
    float* cval;
    uint32_t run;   // candidates written so far
    double ssd;
    int ncf;
    uint32_t s0, s1;  // Random-k keys
    uint32_t pz;      // first pass: keys >= pz leave +0 in the residual instead of acc (NONE: none)
    uint32_t nb;      // bins of the histogram in use: a key whose bin number is nb or more counts as above the bracket
};

__device__ __forceinline__ void cand_hist(TileCtx& c, uint32_t key)
{
#pragma unroll
    for (int j = 0; j < MAXCF; ++j) {
        if (j < c.ncf && key >= c.lo[j]) {
            const uint32_t b = (key - c.lo[j]) >> c.sh[j];
            if (b >= c.nb) c.ovf[j]++;
            else atomicAdd(&c.h1[j * REP * NBIN + b], 1u);
        }
    }
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
template <bool RND>
__device__ __forceinline__ void keys_of_row(const TileCtx& c, const float a[4], int64_t g, uint32_t key[4])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) key[e] = RND ? priority_of(c.s0, c.s1, (uint32_t)(g + e)) : key_of(a[e]);
}

// One lane's four consecutive elements a[0..3] with keys key[0..3] at global index g; vm = validity bits.
template <bool SSD, bool RND>
__device__ __forceinline__ void consume(TileCtx& c, const float a[4], const uint32_t key[4], int64_t g, unsigned vm)
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
    const bool any = f[0] | f[1] | f[2] | f[3];
    if (__ballot(any) != 0ull) {
        uint32_t pre = 0, tot = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t m = __ballot(f[e]);
            pre += lanes_below(m);
            tot += (uint32_t)__popcll(m);
        }
        uint32_t w = c.run + pre;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (f[e]) {
                c.cidx[w] = (int32_t)(g + e);
                c.cval[w] = a[e];
                ++w;
                cand_hist(c, key[e]);
            }
        }
        c.run += tot;
    }
}

// Modes of the streaming pass.
enum { SM_EF = 0,      // acc = residual + grad, written back into residual
       SM_EXACT = 1,   // exact route: acc is re-read, candidates are collected again
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

// Arithmetic and stores of one row; a[] gets the four acc values.
template <int M>
__device__ __forceinline__ void row_finish(const Params& p, int64_t g, const v4f& x, const v4f& y, const v4i& m, float a[4])
{
    if (M == SM_EF) {
        const v4f av = x + y;  // stored by store_acc_row, once the keys are known
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

// First pass: acc goes back into the residual, except that an entry whose key lies above the committed CF's
// bracket leaves +0 there already: it is selected unless the bound fails (the candidate lists keep its value, and
// the routes for a failed bound put it back where it turns out not to be selected), which spares the emit step
// a scattered store per selected entry.
__device__ __forceinline__ void store_acc_row(const Params& p, const TileCtx& c, int64_t g, const float a[4], const uint32_t key[4])
{
    v4f o;
    o.x = key[0] >= c.pz ? 0.0f : a[0];
    o.y = key[1] >= c.pz ? 0.0f : a[1];
    o.z = key[2] >= c.pz ? 0.0f : a[2];
    o.w = key[3] >= c.pz ? 0.0f : a[3];
    st_stream(o, (v4f*)(p.res + g));
}

// Exact route: the bounds of the segment a wavefront last worked on (they cost a histogram search).
struct ExactBounds {
    int t;  // segment, -1 = none yet
    uint32_t lo[MAXCF];
    uint32_t sh[MAXCF];
    uint32_t lo_min;
};

// One sub-tile v, by one wavefront.
template <int M, bool RND>
__device__ __forceinline__ void stream_subtile(const Params& p, uint32_t v, int lane, ExactBounds* xb)
{
    constexpr bool EF = (M != SM_EXACT);  // a first pass: sums acc^2, takes the bounds from the threshold kernel
    const uint32_t u = v / SUB;  // tile
    if (u >= p.n_tiles) return;
    const int t = tile_seg(p, u);
    const uint32_t fail_kind = EF ? (uint32_t)FAIL_NONE : p.seg[t].fail;
    if (!EF && fail_kind == FAIL_NONE) return;
    const int64_t sb = seg_begin(p, t), se = seg_end(p, t);
    const int64_t s0 = sb + (int64_t)(u - seg_tile0(p, t)) * TW + (int64_t)(v % SUB) * TS;
    const int64_t e0 = (s0 + TS < se) ? s0 + TS : se;
    if (s0 >= se) {  // sub-tile past the end of the segment
        if (lane == 0) { p.cand_cnt[v] = 0; if (EF) p.ssd[v] = 0.0; }
        return;
    }

    TileCtx c;
    c.ncf = p.n_cf;
    c.s0 = p.rk_s0; c.s1 = p.rk_s1;
    c.lo_min = NONE;
#pragma unroll
    for (int j = 0; j < MAXCF; ++j) {
        c.ovf[j] = 0;
        c.lo[j] = NONE;
        c.sh[j] = 0;
    }
    c.pz = NONE;
    // The exact route bins one coarse bin (or one bin of the first histogram) into 1024 parts: what lies above it
    // needs no bin of its own, and half of the histogram updates with it.
    c.nb = EF ? OVF : 1024u;
    if (EF) {
        c.lo_min = p.seg[t].lo_min;
        if (M == SM_EF) c.pz = p.seg[t].pz;
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) {
            if (j < p.n_cf) {
                c.lo[j] = p.st[(size_t)t * p.n_cf + j].lo;
                c.sh[j] = p.st[(size_t)t * p.n_cf + j].s;
            }
        }
    } else {
        // exact route: lo_j = base of the coarse (key >> 20) bin that holds the k_j-th largest; 1024 bins of
        // 2^10 keys cover that coarse bin, keys above it land in the open last bin
        const bool first = (v == seg_tile0(p, t) * SUB);
        if (xb->t != t) {
            xb->t = t;
            xb->lo_min = NONE;
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) {
                xb->lo[j] = NONE;
                xb->sh[j] = 10;
                if (j < p.n_cf) {
                    if (fail_kind == FAIL_NARROW) {
                        // the locate step has left the bounds of the CFs that are binned again; the others keep
                        // their histogram and their plan (lo = NONE: no key is counted for them here)
                        const CfState* st = &p.st[(size_t)t * p.n_cf + j];
                        if (st->redo) { xb->lo[j] = st->lo2; xb->sh[j] = st->s2; }
                    } else {
                        uint32_t b, ab, cn;
                        wave_locate_bin(p.coarse + (size_t)t * NBIN, 1, nullptr, seg_k(p, t, j), b, ab, cn);
                        if (b == NONE) { b = 0; if (lane == 0) p.status->error = 1; }
                        xb->lo[j] = b << 20;
                    }
                    xb->lo_min = xb->lo[j] < xb->lo_min ? xb->lo[j] : xb->lo_min;
                }
            }
        }
        c.lo_min = xb->lo_min;
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) {
            if (j < p.n_cf) {
                c.lo[j] = xb->lo[j];
                c.sh[j] = xb->sh[j];
                if (first && c.lo[j] != NONE) {
                    // record the new bound; clear what the refine pass may add to
                    CfState* st = &p.st[(size_t)t * p.n_cf + j];
                    if (lane == 0) { st->lo = c.lo[j]; st->s = c.sh[j]; st->mode = MODE_FAIL; st->redo = 1; }
                    for (int i = lane; i < NBIN; i += 64) p.hist2[((size_t)t * p.n_cf + j) * NBIN + i] = 0;
                    if (lane < REP) p.list_cnt[(((size_t)t * p.n_cf + j) * REP + lane) * 32] = 0;
                }
            }
        }
        // (on the narrow route the candidate lists and the segment's candidate threshold stay as they are)
        if (first && lane == 0 && fail_kind != FAIL_NARROW) p.seg[t].lo_min = c.lo_min;
    }
    // the copy of the histogram this wavefront adds to: spread by the sub-tile number, and by the tile number too,
    // because the exact route's re-binning calls arrive with v = 8 u only
    c.h1 = p.hist1 + ((size_t)t * p.n_cf * REP + ((v ^ (v / SUB)) & (REP - 1))) * NBIN;
    c.cidx = p.cand_idx + (size_t)v * TS;
    c.cval = p.cand_val + (size_t)v * TS;
    c.run = 0;
    c.ssd = 0.0;

    if (!EF && fail_kind != FAIL_FULL) {
        // the candidate lists stay as they are; only their histogram is rebuilt with the new bins.  Called for the
        // first sub-tile of a tile only: the wavefront takes the candidates of the whole tile
        const TileCands tcs = tile_cands(p, u);
        const uint32_t cnt = tcs.total();
        const float* cv = p.cand_val + (size_t)u * TW;
        const int32_t* ci = p.cand_idx + (size_t)u * TW;
        for (uint32_t i0 = 0; i0 < cnt; i0 += 64 * 8) {
            uint32_t kq[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t i = i0 + q * 64 + lane;
                const uint32_t sl = (i < cnt) ? tcs.slot(i) : 0u;
                kq[q] = RND ? priority_of(c.s0, c.s1, (uint32_t)ci[sl]) : key_of(cv[sl]);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (i0 + q * 64 + lane < cnt) cand_hist(c, kq[q]);
        }
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) {
            if (j < p.n_cf) {
                const uint32_t o = wave_sum(c.ovf[j]);
                if (lane == 0 && o) atomicAdd(&p.ovfc[(((size_t)t * p.n_cf + j) * 64 + (u & 63)) * 32], o);
            }
        }
        return;
    }

    // rows start at a multiple of 4 elements so that vector accesses are 16-byte aligned
    for (int64_t rb = s0 & ~(int64_t)3; rb < e0; rb += ROW) {
        const bool full = (rb >= s0) && (rb + ROW <= e0);
        if (full && rb + GV_ROWS * ROW <= e0) {
            // GV_ROWS full rows: all loads first, then the arithmetic
            v4f x[GV_ROWS], y[GV_ROWS];
            v4i m[GV_ROWS];
#pragma unroll
            for (int q = 0; q < GV_ROWS; ++q) row_load<M>(p, rb + q * ROW + 4 * lane, x[q], y[q], m[q]);
#pragma unroll
            for (int q = 0; q < GV_ROWS; ++q) {
                const int64_t g = rb + q * ROW + 4 * lane;
                float a[4];
                uint32_t key[4];
                row_finish<M>(p, g, x[q], y[q], m[q], a);
                keys_of_row<RND>(c, a, g, key);
                if (M == SM_EF) store_acc_row(p, c, g, a, key);
                consume<EF, RND>(c, a, key, g, 0xFu);
            }
            rb += (GV_ROWS - 1) * ROW;
        } else if (full) {
            const int64_t g = rb + 4 * lane;
            v4f x, y;
            v4i m;
            float a[4];
            uint32_t key[4];
            row_load<M>(p, g, x, y, m);
            row_finish<M>(p, g, x, y, m, a);
            keys_of_row<RND>(c, a, g, key);
            if (M == SM_EF) store_acc_row(p, c, g, a, key);
            consume<EF, RND>(c, a, key, g, 0xFu);
        } else {
            // ragged row: element-wise, guarded
            const int64_t g = rb + 4 * lane;
            float a[4];
            unsigned vm = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t q = g + e;
                a[e] = 0.0f;
                if (q >= s0 && q < e0) {
                    vm |= 1u << e;
                    if (M == SM_EF) {
                        a[e] = p.res[q] + p.grad[q];  // stored below, once the keys are known
                    } else if (M == SM_EXACT) {
                        a[e] = p.acc[q];
                    } else {
                        a[e] = p.grad[q];
                        if (p.restore) {
                            const int mi = p.map_idx[q];
                            if ((uint64_t)(int64_t)mi < (uint64_t)p.n_restore) p.restore[mi] = a[e];
                        }
                    }
                }
            }
            uint32_t key[4];
            keys_of_row<RND>(c, a, g, key);
            if (M == SM_EF) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((vm >> e) & 1u) p.res[g + e] = key[e] >= c.pz ? 0.0f : a[e];
            }
            consume<EF, RND>(c, a, key, g, vm);
        }
    }

#pragma unroll
    for (int j = 0; j < MAXCF; ++j) {
        if (j < p.n_cf) {
            const uint32_t o = wave_sum(c.ovf[j]);
            if (lane == 0 && o) atomicAdd(&p.ovfc[(((size_t)t * p.n_cf + j) * 64 + (v & 63)) * 32], o);
        }
    }
    if (EF) {
        const double s = wave_sum(c.ssd);
        if (lane == 0) p.ssd[v] = s;
    }
    if (lane == 0) p.cand_cnt[v] = c.run;
}

// First pass (SM_EF, SM_SINGLE): one sub-tile per wavefront, one launch covers the whole gradient.
// SM_EXACT: a fixed number of wavefronts walks over all tiles (only those of failed segments do any work).
template <int M, bool RND>
__global__ __launch_bounds__(WG) void stream_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t w = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + (threadIdx.x >> 6));
    if (M != SM_EXACT) {
        stream_subtile<M, RND>(p, w, lane, nullptr);
    } else {
        if (p.status->any_fail == 0) return;
        ExactBounds xb;
        xb.t = -1;
        const uint32_t nw = gridDim.x * WAVES;
        for (uint32_t u = w; u < p.n_tiles; u += nw) {
            const uint32_t kind = p.seg[tile_seg(p, u)].fail;
            if (kind == FAIL_NONE) continue;
            // FAIL_NARROW, FAIL_LIGHT: one call re-bins the candidates of the whole tile; FAIL_FULL: sub-tile by sub-tile
            const int subs = (kind == FAIL_FULL) ? SUB : 1;
            for (int j = 0; j < subs; ++j) stream_subtile<SM_EXACT, RND>(p, u * SUB + j, lane, &xb);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// F1 (exact route): histogram of key >> 20 over the tiles of failed segments; the wavefront of a
// failed segment's first tile also clears that segment's candidate histograms
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
            if (kind == FAIL_NARROW) {
                // no coarse histogram: the wavefront of the segment's first tile clears the candidate histograms of
                // the CFs that are binned again
                const uint32_t u = ub + (tid >> 6);
                if (u < ue && u == seg_tile0(p, t)) {
                    for (int j = 0; j < p.n_cf; ++j) {
                        if (p.st[(size_t)t * p.n_cf + j].redo == 0) continue;
                        for (int i = lane; i < REP * NBIN; i += 64) p.hist1[((size_t)t * p.n_cf + j) * REP * NBIN + i] = 0;
                        p.ovfc[(((size_t)t * p.n_cf + j) * 64 + lane) * 32] = 0;
                    }
                }
            } else if (kind != FAIL_NONE) {
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
                        for (int i = lane; i < p.n_cf * REP * NBIN; i += 64) p.hist1[(size_t)t * p.n_cf * REP * NBIN + i] = 0;
                        for (int i = lane; i < p.n_cf * 64; i += 64) p.ovfc[((size_t)t * p.n_cf * 64 + i) * 32] = 0;
                    }
                    if (kind == FAIL_LIGHT) {
                        // the candidates of the tile are enough
                        const TileCands tcs = tile_cands(p, u);
                        const float* cv = p.cand_val + (size_t)u * TW;
                        const int32_t* ci = p.cand_idx + (size_t)u * TW;
                        const uint32_t cnt = tcs.total();
                        for (uint32_t i0 = 0; i0 < cnt; i0 += 64 * 8) {
                            // eight loads in flight per lane (an absent candidate reads slot 0 and is not counted)
                            float vq[8];
                            int32_t iq[8];
#pragma unroll
                            for (int q = 0; q < 8; ++q) {
                                const uint32_t i = i0 + q * 64 + lane;
                                const uint32_t sl = (i < cnt) ? tcs.slot(i) : 0u;
                                vq[q] = cv[sl];
                                iq[q] = p.random ? ci[sl] : 0;
                            }
#pragma unroll
                            for (int q = 0; q < 8; ++q)
                                if (i0 + q * 64 + lane < cnt) atomicAdd(&h[cand_key(p, iq[q], vq[q]) >> 20], 1u);
                        }
                    } else {
                        const uint32_t pz = p.single ? NONE : p.seg[t].pz;
                        if (pz != NONE) {
                            // acc is read again from the residual: first put back what the first pass replaced by +0 in
                            // this tile (the tile's candidate lists hold those values; nobody else touches the tile)
                            const TileCands tcs = tile_cands(p, u);
                            const float* cv = p.cand_val + (size_t)u * TW;
                            const int32_t* ci = p.cand_idx + (size_t)u * TW;
                            const uint32_t cnt = tcs.total();
                            for (uint32_t i0 = 0; i0 < cnt; i0 += 64 * 8) {
                                float vq[8];
                                int32_t iq[8];
#pragma unroll
                                for (int q = 0; q < 8; ++q) {
                                    const uint32_t i = i0 + q * 64 + lane;
                                    const uint32_t sl = (i < cnt) ? tcs.slot(i) : 0u;
                                    vq[q] = cv[sl];
                                    iq[q] = ci[sl];
                                }
#pragma unroll
                                for (int q = 0; q < 8; ++q)
                                    if (i0 + q * 64 + lane < cnt && cand_key(p, iq[q], vq[q]) >= pz) p.res[iq[q]] = vq[q];
                            }
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
    uint32_t mode, base, open, above, c;
};

// Decide from the located bin (b, above, c) of the candidate histogram with bins (key - lo) >> s.
__device__ __forceinline__ BinPlan plan_bin(uint32_t lo, uint32_t s, uint32_t b, uint32_t above, uint32_t c)
{
    BinPlan q;
    if (b == NONE) q.mode = MODE_FAIL;  // fewer than k candidates: the bound was too high
    else if (b == OVF) q.mode = (c <= LCAP) ? MODE_GATHER : MODE_FAIL;
    else if (s == 0) q.mode = MODE_RESOLVED;
    else if (c <= LCAP) q.mode = MODE_GATHER;
    else if (s <= 11) q.mode = MODE_HIST;
    else q.mode = MODE_FAIL;
    q.base = (b == NONE) ? 0u : lo + (b << s);
    q.open = (b == OVF) ? 1u : 0u;
    q.above = above;
    q.c = c;
    return q;
}

__device__ __forceinline__ void store_plan(CfState* st, const BinPlan& q)
{
    st->mode = q.mode;
    if (q.mode != MODE_FAIL) {
        st->base = q.base; st->open = q.open; st->above = q.above; st->c = q.c;
        if (q.mode == MODE_RESOLVED) { st->tau = q.base; st->cnt_gt = q.above; st->need = st->k - q.above; }
    }
}

// ---------------------------------------------------------------------------------------------
// L1: one workgroup per (segment, CF): find the candidate-histogram bin of the k-th largest and
// decide how to resolve it; a segment whose bound failed is marked for the exact route
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void locate_kernel(Params p)
{
    __shared__ uint32_t scratch[8];
    const int tid = threadIdx.x;
    const uint32_t id = blockIdx.x;
    const int t = id / p.n_cf;
    CfState* st = &p.st[id];
    uint32_t b, above, c;
    team_locate_bin(p.hist1 + (size_t)id * REP * NBIN, REP, p.ovfc + (size_t)id * 64 * 32, st->k, tid, scratch,
                    [] { __syncthreads(); }, b, above, c);
    const BinPlan q = plan_bin(st->lo, st->s, b, above, c);
    if (q.mode == MODE_HIST)
        for (int i = tid; i < NBIN; i += 256) p.hist2[(size_t)id * NBIN + i] = 0;
    if (tid == 0) {
        store_plan(st, q);
        if (q.mode == MODE_FAIL) {
            p.status->any_fail = 1;
            uint32_t kind = FAIL_FULL;               // fewer than k candidates
            if (b == OVF) kind = FAIL_LIGHT;         // above the bracket, more keys there than a gather list holds
            else if (b != NONE) {
                // a bin 2^s keys wide (s > 11) with more than LCAP keys: 1024 bins of 2^(s - 10) keys cover it, and a
                // bin at most 2^10 keys wide can always be resolved (gathered or histogrammed key by key)
                kind = FAIL_NARROW;
                st->redo = 1; st->lo2 = q.base; st->s2 = st->s - 10;
            }
            if (atomicMax(&p.seg[t].fail, kind) == 0u) atomicAdd(&p.status->n_fail, 1);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// R1: one pass over the candidates: gather (or histogram) the keys of the bin that holds the
// k-th largest.  For a segment that took the exact route the plan is derived here, by every
// wavefront for itself, from the rebuilt candidate histogram (its first tile's wavefront records it).
// ---------------------------------------------------------------------------------------------
template <int NCF>  // compiled for calls with up to NCF CFs: the loops over the CFs are unrolled
__global__ __launch_bounds__(LWG) void refine_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t u = __builtin_amdgcn_readfirstlane(blockIdx.x * LWAVES + (threadIdx.x >> 6));
    if (u >= p.n_tiles) return;
    const TileCands tc = tile_cands(p, u);
    const uint32_t cnt = tc.total();
    const int t = tile_seg(p, u);
    const bool redo = p.status->any_fail != 0 && p.seg[t].fail != 0;
    const bool first = redo && (u == seg_tile0(p, t));
    if (cnt == 0 && !first) return;
    // exact route: the plan comes from the rebuilt candidate histogram.  A plain loop whose results go through
    // LDS, so that the search does not inflate the register count of the common path.
    __shared__ uint32_t rp[LWAVES][MAXCF][3];
    const int wib = threadIdx.x >> 6;
    if (redo) {
        const uint32_t fail_kind = p.seg[t].fail;
        if (first && lane == 0 && fail_kind != FAIL_FULL) atomicAdd(&p.status->n_light, 1);
        for (int j = 0; j < p.n_cf; ++j) {
            CfState* st = &p.st[(size_t)t * p.n_cf + j];
            if (fail_kind == FAIL_NARROW && st->redo == 0) {
                // this CF was not binned again: its plan stands (nobody writes it during this kernel)
                if (lane == 0) { rp[wib][j][0] = st->mode; rp[wib][j][1] = st->base; rp[wib][j][2] = st->open; }
                continue;
            }
            uint32_t b, above, c;
            wave_locate_bin(p.hist1 + ((size_t)t * p.n_cf + j) * REP * NBIN, REP, p.ovfc + ((size_t)t * p.n_cf + j) * 64 * 32,
                            st->k, b, above, c);
            const BinPlan q = plan_bin(st->lo, st->s, b, above, c);
            if (lane == 0) {
                rp[wib][j][0] = q.mode; rp[wib][j][1] = q.base; rp[wib][j][2] = q.open;
                if (first) {
                    store_plan(st, q);
                    if (q.mode == MODE_FAIL) p.status->error = 1;  // the exact route cannot fail
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");  // rp is read back by the same wavefront
    }
    uint32_t mode[NCF], base[NCF], span[NCF];
    bool work = false;
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        mode[j] = MODE_RESOLVED; base[j] = 0; span[j] = 0;
        if (j < p.n_cf) {
            const CfState* st = &p.st[(size_t)t * p.n_cf + j];
            const uint32_t s = st->s;
            uint32_t open;
            if (redo) { mode[j] = rp[wib][j][0]; base[j] = rp[wib][j][1]; open = rp[wib][j][2]; }
            else { mode[j] = st->mode; base[j] = st->base; open = st->open; }
            span[j] = open ? NONE : ((1u << s) - 1u);  // in the bin <=> key - base <= span
            work |= (mode[j] == MODE_GATHER || mode[j] == MODE_HIST);
        }
    }
    if (!work || cnt == 0) return;
    const float* cv = p.cand_val + (size_t)u * TW;
    const int32_t* ci = p.cand_idx + (size_t)u * TW;
    // what one candidate key adds, per CF, if it lies in the bin that holds the k-th largest
    const auto take = [&](uint32_t key, bool live) {
#pragma unroll
        for (int j = 0; j < NCF; ++j) {
            if (j >= p.n_cf) continue;
            const bool in = live && key >= base[j] && key - base[j] <= span[j];
            if (mode[j] == MODE_GATHER) {
                // one counter update per wavefront: the lanes with a key in the bin take consecutive slots
                const uint64_t m = __ballot(in);
                if (m != 0ull) {
                    const size_t lst = ((size_t)t * p.n_cf + j) * REP + (blockIdx.x & (REP - 1));
                    const int leader = __ffsll((unsigned long long)m) - 1;
                    uint32_t first = 0;
                    if (lane == leader) first = atomicAdd(&p.list_cnt[lst * 32], (uint32_t)__popcll(m));
                    first = __shfl(first, leader, 64);
                    const uint32_t pos = first + lanes_below(m);
                    if (in && pos < LCAP) p.list[lst * LCAP + pos] = key;
                }
            } else if (mode[j] == MODE_HIST && in) {
                atomicAdd(&p.hist2[((size_t)t * p.n_cf + j) * NBIN + (key - base[j])], 1u);
            }
        }
    };
    if (cnt < DENSE_TILE) {
        for (uint32_t i0 = 0; i0 < cnt; i0 += 64 * 8) {
            // eight loads in flight per lane
            uint32_t kq[8];
            if (p.random) {  // the key comes from the index: all loads first, then the arithmetic
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const uint32_t i = i0 + q * 64 + lane;
                    kq[q] = (uint32_t)ci[(i < cnt) ? tc.slot(i) : 0u];
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) kq[q] = priority_of(p.rk_s0, p.rk_s1, kq[q]);
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const uint32_t i = i0 + q * 64 + lane;
                    kq[q] = key_of(cv[(i < cnt) ? tc.slot(i) : 0u]);
                }
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) take(kq[q], i0 + q * 64 + lane < cnt);
        }
        return;
    }
    {
        // a dense tile: four consecutive slots per lane and load, the same VCHUNK slots of VLISTS lists in flight
        // together (see count_kernel)
        const v4f* cv4 = (const v4f*)cv;
        const v4i* ci4 = (const v4i*)ci;
        const uint32_t nmax = tc.longest();
        for (uint32_t c0 = 0; c0 < nmax; c0 += VCHUNK) {
            const uint32_t first = c0 + 4 * lane;  // < TS
            // (the forms for many CFs are too long for this loop to be unrolled: they read the list counts from memory,
            // not from the register array, which can only be indexed by constants)
#pragma unroll
            for (int j0 = 0; j0 < SUB; j0 += VLISTS) {
                v4i kv[VLISTS];  // the bits the key is made from: the value's, or the index for Random-k
                if (p.random) {
#pragma unroll
                    for (int j = 0; j < VLISTS; ++j) kv[j] = ci4[(j0 + j) * (TS / 4) + first / 4];
                } else {
#pragma unroll
                    for (int j = 0; j < VLISTS; ++j) kv[j] = __builtin_bit_cast(v4i, cv4[(j0 + j) * (TS / 4) + first / 4]);
                }
#pragma unroll
                for (int j = 0; j < VLISTS; ++j) {
                    uint32_t n;
                    if constexpr (NCF <= 2) n = tc.start[j0 + j + 1] - tc.start[j0 + j];
                    else n = p.cand_cnt[(size_t)u * SUB + j0 + j];
                    if (n <= c0) continue;  // the same for all lanes
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        take(p.random ? priority_of(p.rk_s0, p.rk_s1, (uint32_t)kv[j][x]) : ((uint32_t)kv[j][x] & 0x7FFFFFFFu),
                             first + x < n);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// L2: per (segment, CF) resolve the exact key tau of the k-th largest, and how many ties it takes
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void resolve_kernel(Params p)
{
    __shared__ uint32_t wsum[2][WAVES];
    const int id = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    CfState* st = &p.st[id];
    // the fill counts of the gather lists are fetched together with the plan, not after it (they do not depend on it)
    uint32_t fill[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) fill[r] = p.list_cnt[((size_t)id * REP + r) * 32];
    const uint32_t mode = st->mode;
    if (mode == MODE_RESOLVED) return;
    if (mode == MODE_FAIL) { if (tid == 0) p.status->error = 1; return; }
    const uint32_t k = st->k, above = st->above, want = k - above;  // want-th largest inside the bin
    const uint32_t base = st->base;
    if (mode == MODE_HIST) {
        if (wib != 0) return;
        uint32_t b, ab, cn;  // bins are single keys: base + b
        wave_locate_bin(p.hist2 + (size_t)id * NBIN, 1, nullptr, want, b, ab, cn);
        if (lane == 0) {
            if (b == NONE) { p.status->error = 1; b = 0; }
            st->tau = base + b;
            st->cnt_gt = above + ab;
            st->need = k - st->cnt_gt;
            st->mode = MODE_RESOLVED;
        }
        return;
    }
    // gather: the want-th largest of the listed keys, by a bitwise search on d = key - base.
    // The keys sit in REP lists; list r holds positions [off_r, off_r + n_r) of the concatenation.
    const uint32_t c = st->c;
    uint32_t off[REP + 1];
    off[0] = 0;
#pragma unroll
    for (int r = 0; r < REP; ++r) off[r + 1] = off[r] + fill[r];
    if (off[REP] != c || c > LCAP || want == 0 || want > c) { if (tid == 0) p.status->error = 1; return; }
    uint32_t d[LCAP / 256];
    // all loads first, without branches around them (a position past the last key reads key 0 of the lists
    // instead; c >= 1 here), so that they are in flight together
#pragma unroll
    for (int q = 0; q < LCAP / 256; ++q) {
        const uint32_t i = (uint32_t)(q * 256 + tid) < c ? (uint32_t)(q * 256 + tid) : 0u;
        int r = 0;
#pragma unroll
        for (int x = 1; x < REP; ++x) r += (i >= off[x]);
        uint32_t o = 0;
#pragma unroll
        for (int x = 0; x < REP; ++x) if (x == r) o = off[x];
        d[q] = p.list[((size_t)id * REP + r) * LCAP + (i - o)];
    }
#pragma unroll
    for (int q = 0; q < LCAP / 256; ++q)
        d[q] = (uint32_t)(q * 256 + tid) < c ? d[q] - base : 0u;  // padding never counts: trial values are >= 1
    const int nbits = st->open ? 31 : (int)st->s;
    uint32_t prefix = 0;
    int buf = 0;
    for (int bit = nbits - 1; bit >= 0; --bit) {
        const uint32_t trial = prefix | (1u << bit);
        uint32_t cnt = 0;
#pragma unroll
        for (int q = 0; q < LCAP / 256; ++q) cnt += (d[q] >= trial);
        cnt = wave_sum(cnt);
        if (lane == 0) wsum[buf][wib] = cnt;
        __syncthreads();
        const uint32_t total = wsum[buf][0] + wsum[buf][1] + wsum[buf][2] + wsum[buf][3];
        buf ^= 1;
        if (total >= want) prefix = trial;
    }
    uint32_t gt = 0;
#pragma unroll
    for (int q = 0; q < LCAP / 256; ++q) gt += (q * 256 + tid < c) && (d[q] > prefix);
    gt = wave_sum(gt);
    __syncthreads();
    if (lane == 0) wsum[0][wib] = gt;
    __syncthreads();
    if (tid == 0) {
        st->tau = base + prefix;
        st->cnt_gt = above + wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
        st->need = k - st->cnt_gt;
        st->mode = MODE_RESOLVED;
    }
}

// ---------------------------------------------------------------------------------------------
// K3: one wavefront per tile: candidates above / at the committed threshold, energy above each
// CF's threshold.  Written for every tile, so that the scan needs no second look at cand_cnt.
// ---------------------------------------------------------------------------------------------
template <int NCF>  // as refine_kernel
__global__ __launch_bounds__(LWG) void count_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t u = __builtin_amdgcn_readfirstlane(blockIdx.x * LWAVES + (threadIdx.x >> 6));
    if (u >= p.n_tiles) return;
    const TileCands tcs = tile_cands(p, u);
    const uint32_t cnt = tcs.total();
    {   // energy of the tile = sum over its sub-tiles, in a fixed order
        const double x = wave_sum(lane < SUB ? p.ssd[(size_t)u * SUB + lane] : 0.0);
        if (lane == 0) p.ssd_t[u] = x;
    }
    if (cnt == 0) {
        if (lane == 0) { p.tg[u] = 0; p.te[u] = 0; }
        if (lane < p.n_cf) p.sss[(size_t)u * p.n_cf + lane] = 0.0;
        return;
    }
    const int t = tile_seg(p, u);
    uint32_t tau[NCF];
    uint32_t tc = 0;
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        tau[j] = (j < p.n_cf) ? p.st[(size_t)t * p.n_cf + j].tau : NONE;
        if (j == p.commit) tc = tau[j];
    }
    double ss[NCF];
#pragma unroll
    for (int j = 0; j < NCF; ++j) ss[j] = 0.0;
    uint32_t g = 0, e = 0;
    const float* cv = p.cand_val + (size_t)u * TW;
    const int32_t* ci = p.cand_idx + (size_t)u * TW;
    // Random-k: priorities are distinct, the entry at the threshold is the last one selected and has no
    // particular magnitude, so its energy is summed here (Top-k adds need * tau^2 in the scan instead)
    const uint32_t at_tau = p.random ? 1u : 0u;
    if (cnt < DENSE_TILE) {
        for (uint32_t i0 = 0; i0 < cnt; i0 += 64 * 8) {
            float vq[8];
            uint32_t kq[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t i = i0 + q * 64 + lane;
                const uint32_t sl = (i < cnt) ? tcs.slot(i) : 0u;
                vq[q] = cv[sl];
                kq[q] = p.random ? (uint32_t)ci[sl] : 0u;   // all loads first, then the arithmetic
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) kq[q] = p.random ? priority_of(p.rk_s0, p.rk_s1, kq[q]) : key_of(vq[q]);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (i0 + q * 64 + lane < cnt) {
                    const uint32_t key = kq[q];
                    const double dv = (double)vq[q];
                    g += (key > tc);
                    e += (key == tc);
#pragma unroll
                    for (int j = 0; j < NCF; ++j) if (j < p.n_cf && key + at_tau > tau[j]) ss[j] += dv * dv;
                }
            }
        }
    } else {
        // A dense tile: four consecutive slots per lane and load, the same VCHUNK slots of VLISTS lists in flight
        // together (a list of TS slots is aligned to 16 bytes; slots past a list's count hold older entries and
        // are masked off).  A sparse tile would leave most lanes of such a walk idle and takes the loop below.
        const v4f* cv4 = (const v4f*)cv;
        const v4i* ci4 = (const v4i*)ci;
        const uint32_t nmax = tcs.longest();
        static_assert(SUB % VLISTS == 0, "the lists are taken VLISTS at a time");
        for (uint32_t c0 = 0; c0 < nmax; c0 += VCHUNK) {
            const uint32_t first = c0 + 4 * lane;  // < TS
#pragma unroll
            for (int j0 = 0; j0 < SUB; j0 += VLISTS) {
                v4f v[VLISTS];
                v4i ix[VLISTS];
#pragma unroll
                for (int j = 0; j < VLISTS; ++j) v[j] = cv4[(j0 + j) * (TS / 4) + first / 4];
                if (p.random) {
#pragma unroll
                    for (int j = 0; j < VLISTS; ++j) ix[j] = ci4[(j0 + j) * (TS / 4) + first / 4];
                }
#pragma unroll
                for (int j = 0; j < VLISTS; ++j) {
                    const uint32_t n = tcs.start[j0 + j + 1] - tcs.start[j0 + j];
                    if (n <= c0) continue;  // the same for all lanes
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const bool live = first + x < n;
                        const uint32_t key = p.random ? priority_of(p.rk_s0, p.rk_s1, (uint32_t)ix[j][x]) : key_of(v[j][x]);
                        const double dv = (double)v[j][x];
                        g += (live && key > tc);
                        e += (live && key == tc);
#pragma unroll
                        for (int c = 0; c < NCF; ++c) if (c < p.n_cf && live && key + at_tau > tau[c]) ss[c] += dv * dv;
                    }
                }
            }
        }
    }
    g = wave_sum(g);
    e = wave_sum(e);
#pragma unroll
    for (int j = 0; j < NCF; ++j) {
        if (j < p.n_cf) {
            const double x = wave_sum(ss[j]);
            if (lane == 0) p.sss[(size_t)u * p.n_cf + j] = x;
        }
    }
    if (lane == 0) { p.tg[u] = g; p.te[u] = e; }
}

// ---------------------------------------------------------------------------------------------
// SCAN: grid (n_seg, slices + n_cf).  Block (t, y < slices): exclusive scan of the counts of the
//       y-th slice of SCAN_SLICE tiles of segment t -> every tile's output offset and tie quota.
//       The totals of the earlier slices are re-added by every block (a few batched loads), so no
//       block waits on another.  Block (t, slices + j): statistics of (segment t, CF j), summed
//       over the tiles in a fixed order.
// ---------------------------------------------------------------------------------------------
constexpr int SCAN_T = 1024;                 // threads
constexpr int SCAN_PER = 4;                  // tiles per thread
constexpr int SCAN_SLICE = SCAN_T * SCAN_PER;

__global__ __launch_bounds__(SCAN_T) void scan_kernel(Params p, uint32_t slices)
{
    __shared__ uint32_t sg[SCAN_SLICE], se[SCAN_SLICE];
    __shared__ uint32_t wt[4][16];
    __shared__ double dred[2][SCAN_T / 64];
    const int tid = threadIdx.x, lane = tid & 63, wib = tid >> 6;
    const int t = blockIdx.x;
    if (blockIdx.y < slices) {
        const uint32_t u0 = seg_tile0(p, t), u1 = seg_tile1(p, t);
        const uint32_t base = u0 + blockIdx.y * SCAN_SLICE;
        if (base >= u1) return;
        const uint32_t need = p.st[(size_t)t * p.n_cf + p.commit].need;
        // this slice, coalesced
        uint32_t og[SCAN_PER], oe[SCAN_PER];
#pragma unroll
        for (int q = 0; q < SCAN_PER; ++q) {
            const uint32_t u = base + q * SCAN_T + tid;
            og[q] = (u < u1) ? p.tg[u] : 0u;
            oe[q] = (u < u1) ? p.te[u] : 0u;
        }
        // totals of the earlier slices of this segment
        uint32_t pg = 0, pe = 0;
        for (uint32_t v0 = u0 + tid; v0 < base; v0 += 32 * SCAN_T) {
            uint32_t xg[32], xe[32];
#pragma unroll
            for (int q = 0; q < 32; ++q) {
                const uint32_t v = v0 + q * SCAN_T;
                xg[q] = (v < base) ? p.tg[v] : 0u;
                xe[q] = (v < base) ? p.te[v] : 0u;
            }
#pragma unroll
            for (int q = 0; q < 32; ++q) { pg += xg[q]; pe += xe[q]; }
        }
        pg = wave_sum(pg);
        pe = wave_sum(pe);
#pragma unroll
        for (int q = 0; q < SCAN_PER; ++q) { sg[q * SCAN_T + tid] = og[q]; se[q * SCAN_T + tid] = oe[q]; }
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
        for (int w = 0; w < 16; ++w) {
            if (w < wib) { run_g += wt[0][w]; run_e += wt[1][w]; }
            run_g += wt[2][w];
            run_e += wt[3][w];
        }
#pragma unroll
        for (int i = 0; i < SCAN_PER; ++i) {
            const uint32_t ties_before = run_e < need ? run_e : need;  // ties selected in earlier tiles
            const uint32_t left = need - ties_before;
            sg[tid * SCAN_PER + i] = run_g + ties_before;               // output offset of the tile
            se[tid * SCAN_PER + i] = left < e[i] ? left : e[i];         // its tie quota
            run_g += g[i];
            run_e += e[i];
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < SCAN_PER; ++q) {
            const uint32_t u = base + q * SCAN_T + tid;
            if (u < u1) { p.toff[u] = sg[q * SCAN_T + tid]; p.ttake[u] = se[q * SCAN_T + tid]; }
        }
        return;
    }
    const int j = blockIdx.y - slices;
    const uint32_t id = (uint32_t)t * p.n_cf + j;
    const uint32_t ua = seg_tile0(p, t), ub = seg_tile1(p, t);
    // sixteen tiles per thread and round, all loads of a round in flight together; fixed summation order
    double sd = 0.0, sj = 0.0;
    for (uint32_t u0 = ua + tid; u0 < ub; u0 += 16 * SCAN_T) {
        double xd[16], xj[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const uint32_t u = u0 + q * SCAN_T;
            xd[q] = (u < ub) ? p.ssd_t[u] : 0.0;
            xj[q] = (u < ub) ? p.sss[(size_t)u * p.n_cf + j] : 0.0;
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) { sd += xd[q]; sj += xj[q]; }
    }
    // every wavefront's sum, then the SCAN_T / 64 of them in order: one barrier, the same order in every run
    {
        const double wd = wave_sum(sd), wj = wave_sum(sj);
        if (lane == 0) { dred[0][wib] = wd; dred[1][wib] = wj; }
    }
    __syncthreads();
    if (tid == 0) {
        const CfState* st = &p.st[id];
        // fourth statistic: the threshold as a magnitude (Top-k) or as a priority (Random-k)
        const double tau = p.random ? (double)st->tau : (double)__uint_as_float(st->tau);
        double ss_dense = 0.0, ss_cand = 0.0;
        for (int w = 0; w < SCAN_T / 64; ++w) { ss_dense += dred[0][w]; ss_cand += dred[1][w]; }
        // Top-k: the ties all have magnitude tau; Random-k: the count pass has summed the entry at the threshold
        const double ss_sel = ss_cand + (p.random ? 0.0 : (double)st->need * tau * tau);
        double* o = p.out_stats + (size_t)id * GRAVAC_STATS_PER_CF;
        o[0] = ss_sel;
        o[1] = ss_dense;
        o[2] = (ss_dense == 0.0) ? 1.0 : ss_sel / ss_dense;
        o[3] = tau;
        if (id == 0) {
            if (p.out_count) *p.out_count = p.total_out;
            p.status->sig_lo = p.sig_lo;  // this call's thresholds can serve as the next call's bounds
            p.status->sig_hi = p.sig_hi;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// K4: one wavefront per tile emits the tile's share of the committed selection in ascending index
//     order and zeroes its residual slots
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(LWG) void emit_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t u = __builtin_amdgcn_readfirstlane(blockIdx.x * LWAVES + (threadIdx.x >> 6));
    if (u >= p.n_tiles) return;
    const TileCands tcs = tile_cands(p, u);
    const uint32_t cnt = tcs.total();
    if (cnt == 0) return;
    const uint32_t take = p.ttake[u];
    const int t = tile_seg(p, u);
    const uint32_t tau = p.st[(size_t)t * p.n_cf + p.commit].tau;
    // The first pass has left +0 in the residual for keys >= pz (not on the full exact route, which has put acc back).
    // Those entries need no store here if they are selected, and get acc back if they are not, which can only be
    // when the threshold turned out to lie at or above pz.
    const uint32_t pz = (p.single || p.seg[t].fail == FAIL_FULL) ? NONE : p.seg[t].pz;
    const bool put_back = pz != NONE && tau >= pz;
    if (p.tg[u] == 0 && take == 0 && !put_back) return;
    const int64_t seg_out = seg_koff(p, t);
    const int64_t lim = seg_out + (int64_t)seg_k(p, t, p.commit);  // end of this segment's message
    int64_t pos = seg_out + (int64_t)p.toff[u];
    uint32_t erun = 0;
    const float* cv = p.cand_val + (size_t)u * TW;
    const int32_t* ci = p.cand_idx + (size_t)u * TW;
    // the loads of the next round are issued before this round is worked on (an absent candidate reads slot 0
    // and is not used), so that a wavefront with a long list does not wait a full round trip per round
    float vn[4];
    int32_t in[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t q = r * 64 + lane;
        const uint32_t sl = (q < cnt) ? tcs.slot(q) : 0u;
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
                const uint32_t sl = (q < cnt) ? tcs.slot(q) : 0u;
                vn[r] = cv[sl];
                in[r] = ci[sl];
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool live = b0 + r * 64 + lane < cnt;
            const uint32_t key = cand_key(p, iq[r], vq[r]);
            const bool gt = live && key > tau, eq = live && key == tau;
            const uint64_t me = __ballot(eq);
            const bool sel = gt || (eq && (erun + lanes_below(me)) < take);
            const uint64_t ms = __ballot(sel);
            if (sel) {
                const int64_t o = pos + lanes_below(ms);
                if (o < lim) {
                    p.out_val[o] = vq[r];
                    if (!p.single) {
                        p.out_idx[o] = iq[r];
                        if (key < pz) p.res[iq[r]] = 0.0f;
                    } else {
                        const int mi = p.map_idx[iq[r]];  // position in the message -> index in the gradient
                        p.out_idx[o] = mi;
                        if (p.restore && (uint64_t)(int64_t)mi < (uint64_t)p.n_restore) p.restore[mi] = 0.0f;
                    }
                } else {
                    p.status->error = 1;  // cannot happen if the counts are consistent; never write out of range
                }
            } else if (put_back && live && key >= pz) {
                p.res[iq[r]] = vq[r];
            }
            pos += __popcll(ms);
            erun += (uint32_t)__popcll(me);
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
                                                         WorkerOffsets wo, int W, int64_t n, float* dense)
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
                        if (pw[q] == w) acc[pj[q]] += pv[q];
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
                                                            const uint32_t* __restrict__ bounds)
{
    __shared__ __attribute__((aligned(16))) float acc[DTILE];
    __shared__ uint32_t blo[DENT], bcnt[DENT];      // first pair and number of pairs, per (tile of the chunk, worker)
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
        }
        __syncthreads();
        for (int i = 0; i < tc; ++i) {
            const int64_t tile = c0 + (int64_t)i * gridDim.x;
            if (tile >= ntile) break;
            const int64_t base = tile * DTILE;
            const int len = (int)((n - base < DTILE) ? n - base : DTILE);
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
                            if (pw[q] == w) acc[pj[q]] += pv[q];
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
// host side
// ---------------------------------------------------------------------------------------------

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t status, tables, tables_bytes, tseg, st, seg, hist1, ovfc, hist2, coarse, list, list_cnt,
        samp_hist, cand_cnt, tg, te, toff, ttake, ssd, ssd_t, sss, cand_idx, cand_val, total;
};

// Upper bounds that depend only on (n, n_seg).
uint64_t max_tiles(int64_t n, int n_seg) { return (uint64_t)((n + TW - 1) / TW) + (uint64_t)n_seg; }

uint64_t max_sample_blocks(int64_t n, int n_seg)
{
    static_assert(DENSE_BLOCKS * SAMPLE_BLOCK <= 2 * SAMPLE_MAX && SAMPLE_MAX_FLAT <= DENSE_BLOCKS * SAMPLE_BLOCK * DENSE_ROUNDS,
                  "the blocks of a dense sample fit as well");
    const uint64_t a = (uint64_t)n_seg * (2 * SAMPLE_MAX / SAMPLE_BLOCK);
    const uint64_t b = (uint64_t)((n + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK) + (uint64_t)n_seg;
    return a < b ? a : b;
}

Layout make_layout(int64_t n, int n_cf, int n_seg)
{
    Layout L;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
    const uint64_t nt = max_tiles(n, n_seg), nsb = max_sample_blocks(n, n_seg);
    const size_t sc = (size_t)n_seg * n_cf;
    L.status = take(sizeof(Status));
    // host-built tables, one piece: SegInfo[n_seg], ktab[n_seg][n_cf], sblock_seg[sample blocks]
    L.tables_bytes = sizeof(SegInfo) * n_seg + sizeof(uint32_t) * sc + sizeof(uint32_t) * nsb;
    L.tables = take(L.tables_bytes);
    L.tseg = take(sizeof(uint32_t) * nt);
    L.st = take(sizeof(CfState) * sc);
    L.seg = take(sizeof(SegState) * n_seg);
    L.hist1 = take(sizeof(uint32_t) * sc * REP * NBIN);
    L.ovfc = take(sizeof(uint32_t) * sc * 64 * 32);
    L.hist2 = take(sizeof(uint32_t) * sc * NBIN);
    L.coarse = take(sizeof(uint32_t) * (size_t)n_seg * NBIN);
    L.list = take(sizeof(uint32_t) * sc * REP * LCAP);
    L.list_cnt = take(sizeof(uint32_t) * sc * REP * 32);
    L.samp_hist = take(sizeof(uint32_t) * nsb * (SBIN / 2));
    L.cand_cnt = take(sizeof(uint32_t) * nt * SUB);
    L.tg = take(sizeof(uint32_t) * nt);
    L.te = take(sizeof(uint32_t) * nt);
    L.toff = take(sizeof(uint32_t) * nt);
    L.ttake = take(sizeof(uint32_t) * nt);
    L.ssd = take(sizeof(double) * nt * SUB);
    L.ssd_t = take(sizeof(double) * nt);
    L.sss = take(sizeof(double) * nt * n_cf);
    L.cand_idx = take(sizeof(int32_t) * nt * TW);
    L.cand_val = take(sizeof(float) * nt * TW);
    L.total = at;
    return L;
}

// samples taken from a segment of nt elements when the CFs range from cf_min to cf_max
uint32_t sample_count(uint64_t nt, double cf_min, double cf_max, bool flat)
{
    // layerwise: the larger of 32 CF_max and 1/64 of the tensor.  A small sample of a large tensor gives a wide
    // bracket: many more candidates than k, and bins so coarse that the keys near the bracket's lower end crowd
    // into a few histogram bins, where their atomics queue up behind each other
    uint64_t target = flat ? (uint64_t)SAMPLE_MAX : (uint64_t)(32.0 * std::ceil(cf_max));
    if (!flat && target < nt / 64) target = nt / 64;
    if (target < 4096) target = 4096;
    if (target > (uint64_t)SAMPLE_MAX) target = SAMPLE_MAX;
    if (flat) {
        // The bracket spans about 10 standard deviations of a sampled rank, which is 10 sqrt(k nt / m) of the tensor's
        // entries for m samples, and every candidate inside it costs the streaming pass a device-wide atomic (about
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
struct StagingSlot {
    char* mem = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool pending = false;  // `done` was recorded and not yet waited for
    bool busy = false;     // being filled by a caller
};
constexpr int STAGING_SLOTS = 8;
StagingSlot g_staging[STAGING_SLOTS];
int g_staging_next = 0;
std::mutex g_staging_mutex;

StagingSlot* staging_acquire(size_t bytes)
{
    std::lock_guard<std::mutex> lock(g_staging_mutex);
    StagingSlot* s = nullptr;
    for (int i = 0; i < STAGING_SLOTS && !s; ++i) {
        StagingSlot* c = &g_staging[(g_staging_next + i) % STAGING_SLOTS];
        if (!c->busy) { s = c; g_staging_next = (g_staging_next + i + 1) % STAGING_SLOTS; }
    }
    if (!s) return nullptr;  // more concurrent callers than slots
    if (!s->done && hipEventCreateWithFlags(&s->done, hipEventDisableTiming) != hipSuccess) return nullptr;
    if (s->pending) {
        if (hipEventSynchronize(s->done) != hipSuccess) return nullptr;
        s->pending = false;
    }
    if (s->cap < bytes) {
        if (s->mem) (void)hipHostFree(s->mem);
        s->mem = nullptr; s->cap = 0;
        const size_t want = bytes < 65536 ? 65536 : bytes + bytes / 2;
        if (hipHostMalloc((void**)&s->mem, want, hipHostMallocDefault) != hipSuccess) { s->mem = nullptr; return nullptr; }
        s->cap = want;
    }
    s->busy = true;
    return s;
}

void staging_release(StagingSlot* s, bool recorded)
{
    std::lock_guard<std::mutex> lock(g_staging_mutex);
    s->pending = recorded;
    s->busy = false;
}

// What this process last asked of each workspace (the signature of the last call issued with it), so that a call
// that wants to reuse thresholds on a workspace whose last call had another shape, or that this process has never
// used, can be told apart on the host: it samples like a call without the flag, which costs one pass, whereas on
// the device the mismatch would only show once the sampling kernel can no longer be launched and every segment
// would take the exact route.  A hint only: the device still checks the signature the last completed call left in
// the workspace.  A small ring; a workspace that has dropped out of it samples once.
struct WorkspaceMemo {
    const void* ws = nullptr;
    uint64_t sig = 0;
};
constexpr int WS_MEMO = 64;
WorkspaceMemo g_ws_memo[WS_MEMO];
int g_ws_memo_next = 0;
std::mutex g_ws_memo_mutex;

// records sig as the last call on ws; returns whether the call before it on ws had the same signature
bool ws_memo_exchange(const void* ws, uint64_t sig)
{
    std::lock_guard<std::mutex> lock(g_ws_memo_mutex);
    for (int i = 0; i < WS_MEMO; ++i) {
        if (g_ws_memo[i].ws == ws) {
            const bool same = g_ws_memo[i].sig == sig;
            g_ws_memo[i].sig = sig;
            return same;
        }
    }
    g_ws_memo[g_ws_memo_next].ws = ws;
    g_ws_memo[g_ws_memo_next].sig = sig;
    g_ws_memo_next = (g_ws_memo_next + 1) % WS_MEMO;
    return false;
}

std::mutex g_prof_mutex;
hipEvent_t g_ev[4];
bool g_ev_ready = false;
bool g_ev_recorded = false;

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
// be replayed: a replay would copy whatever the staging slot holds by then, or re-record the timing events).
static int refuse_capture(hipStream_t stream)
{
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) return GRAVAC_ERR_HIP;
    return cap == hipStreamCaptureStatusNone ? GRAVAC_OK : GRAVAC_ERR_CAPTURE;
}

// The pipeline behind both entry points.  map_idx == null: error-feedback compression of grad + residual.
// map_idx != null: single-source mode, the source is grad alone (a message's values), map_idx its indices,
// restore / n_restore the dense residual that takes the unselected values back (may be null).
static int compress_impl(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                         const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val, int64_t out_capacity,
                         int64_t* out_count, double* out_stats, void* workspace, size_t workspace_bytes, unsigned flags,
                         hipStream_t stream, const int32_t* map_idx, float* restore, int64_t n_restore,
                         const uint64_t* seed)
{
    const bool single = map_idx != nullptr;
    const bool random = seed != nullptr;
    if (random) flags &= ~(unsigned)GRAVAC_FLAG_REUSE_THRESHOLDS;  // the bounds of a random draw need no history
    if (!grad || (!single && !residual) || !cf_list || !out_idx || !out_val || !out_stats) return GRAVAC_ERR_INVALID_ARG;
    if (n <= 0 || n > 2147483647LL || n_cf < 1 || n_cf > MAXCF || commit < 0 || commit >= n_cf) return GRAVAC_ERR_INVALID_ARG;
    if (((uintptr_t)grad & 15) || ((uintptr_t)residual & 15) || ((uintptr_t)map_idx & 15)) return GRAVAC_ERR_INVALID_ARG;
    if (n_seg < 0 || (n_seg > 0 && !seg_offsets) || (int64_t)n_seg > n) return GRAVAC_ERR_INVALID_ARG;
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
    p.n = n; p.n_seg = ns; p.n_cf = n_cf; p.commit = commit; p.flags = flags;
    p.status = (Status*)(ws + L.status);
    p.segs = (const SegInfo*)(ws + L.tables);
    p.ktab = (const uint32_t*)(ws + L.tables + sizeof(SegInfo) * ns);
    p.sblock_seg = p.ktab + (size_t)ns * n_cf;
    p.tseg = (uint32_t*)(ws + L.tseg);
    p.st = (CfState*)(ws + L.st);
    p.seg = (SegState*)(ws + L.seg);
    p.hist1 = (uint32_t*)(ws + L.hist1);
    p.ovfc = (uint32_t*)(ws + L.ovfc);
    p.hist2 = (uint32_t*)(ws + L.hist2);
    p.coarse = (uint32_t*)(ws + L.coarse);
    p.list = (uint32_t*)(ws + L.list);
    p.list_cnt = (uint32_t*)(ws + L.list_cnt);
    p.samp_hist = (uint32_t*)(ws + L.samp_hist);
    p.cand_cnt = (uint32_t*)(ws + L.cand_cnt);
    p.tg = (uint32_t*)(ws + L.tg);
    p.te = (uint32_t*)(ws + L.te);
    p.toff = (uint32_t*)(ws + L.toff);
    p.ttake = (uint32_t*)(ws + L.ttake);
    p.ssd = (double*)(ws + L.ssd);
    p.ssd_t = (double*)(ws + L.ssd_t);
    p.sss = (double*)(ws + L.sss);
    p.cand_idx = (int32_t*)(ws + L.cand_idx);
    p.cand_val = (float*)(ws + L.cand_val);
    p.out_idx = out_idx; p.out_val = out_val; p.out_count = out_count; p.out_stats = out_stats;

    int64_t total_out = 0;
    uint32_t max_seg_tiles = 1;  // tiles of the largest segment
    int sample_rounds = 1;  // groups per thread of the sampling kernel
    uint32_t k_largest = 0;  // over all segments and CFs
    if (ns == 1) {
        for (int j = 0; j < n_cf; ++j) {
            p.flat_k[j] = (uint32_t)gravac_topk_count(n, cf_list[j]);
            if (p.flat_k[j] > k_largest) k_largest = p.flat_k[j];
        }
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
        if (total_out > out_capacity) return GRAVAC_ERR_CAPACITY;
    } else {
        // layerwise tables: sized first, then built straight into a pinned staging slot and copied into the
        // workspace with one asynchronous copy (no host synchronisation)
        uint64_t tiles = 0, sblocks = 0;
        for (int t = 0; t < ns; ++t) {
            const int64_t nt = seg_offsets[t + 1] - seg_offsets[t];
            total_out += gravac_topk_count(nt, cf_list[commit]);
            const uint64_t tt = (uint64_t)((nt + TW - 1) / TW);
            tiles += tt;
            if (tt > max_seg_tiles) max_seg_tiles = (uint32_t)tt;
            sblocks += (sample_count((uint64_t)nt, cf_min, cf_max, false) + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
        }
        if (total_out > out_capacity) return GRAVAC_ERR_CAPACITY;
        if (tiles > max_tiles(n, ns) || sblocks > max_sample_blocks(n, ns)) return GRAVAC_ERR_WORKSPACE;
        if (const int rc = refuse_capture(stream)) return rc;
        p.n_tiles = (uint32_t)tiles;
        p.n_sample_blocks = (uint32_t)sblocks;
        const size_t bytes = sizeof(SegInfo) * ns + sizeof(uint32_t) * (size_t)ns * n_cf + sizeof(uint32_t) * sblocks;
        StagingSlot* slot = staging_acquire(bytes);
        if (!slot) return GRAVAC_ERR_HIP;
        SegInfo* segs = (SegInfo*)slot->mem;
        uint32_t* ktab = (uint32_t*)(slot->mem + sizeof(SegInfo) * ns);
        uint32_t* sblock_seg = ktab + (size_t)ns * n_cf;
        int64_t koff = 0;
        uint32_t tile_at = 0, sb_at = 0;
        for (int t = 0; t < ns; ++t) {
            const int64_t nt = seg_offsets[t + 1] - seg_offsets[t];
            SegInfo& g = segs[t];
            std::memset(&g, 0, sizeof(g));
            g.begin = seg_offsets[t]; g.end = seg_offsets[t + 1]; g.koff = koff;
            g.tile0 = tile_at; tile_at += (uint32_t)((nt + TW - 1) / TW); g.tile1 = tile_at;
            g.samp0 = sb_at; g.samp_cnt = sample_count((uint64_t)nt, cf_min, cf_max, false);
            const uint32_t nb = (g.samp_cnt + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
            for (uint32_t b = 0; b < nb; ++b) sblock_seg[sb_at + b] = (uint32_t)t;
            sb_at += nb;
            for (int j = 0; j < n_cf; ++j) {
                ktab[(size_t)t * n_cf + j] = (uint32_t)gravac_topk_count(nt, cf_list[j]);
                if (ktab[(size_t)t * n_cf + j] > k_largest) k_largest = ktab[(size_t)t * n_cf + j];
            }
            koff += ktab[(size_t)t * n_cf + commit];
        }
        const bool ok = hipMemcpyAsync(ws + L.tables, slot->mem, bytes, hipMemcpyHostToDevice, stream) == hipSuccess &&
                        hipEventRecord(slot->done, stream) == hipSuccess;
        staging_release(slot, ok);
        if (!ok) return GRAVAC_ERR_HIP;
    }

    p.total_out = total_out;
    {   // signature of the call: FNV-1a over the shape, the k table and the segment table
        uint64_t h = 1469598103934665603ull;
        auto mix = [&](uint64_t x) { for (int b = 0; b < 8; ++b) { h ^= (x >> (8 * b)) & 0xFF; h *= 1099511628211ull; } };
        mix((uint64_t)n); mix((uint64_t)n_cf); mix((uint64_t)ns); mix((single ? 1u : 0u) | (random ? 2u : 0u));
        for (int j = 0; j < n_cf; ++j) { uint64_t bits; std::memcpy(&bits, &cf_list[j], 8); mix(bits); }
        if (ns > 1) for (int t = 0; t <= ns; ++t) mix((uint64_t)seg_offsets[t]);
        if (h == 0) h = 1;  // 0 marks "no completed call"
        p.sig_lo = (uint32_t)h; p.sig_hi = (uint32_t)(h >> 32);
        // thresholds can only be reused from a call of the same signature: without one, sample
        if (!ws_memo_exchange(workspace, h)) flags &= ~(unsigned)GRAVAC_FLAG_REUSE_THRESHOLDS;
        p.flags = flags;
    }
    // the sampling pass: always without reuse, and with it for the sake of a CF that selects very many entries
    p.have_sample = (p.n_sample_blocks && !random && (!(flags & GRAVAC_FLAG_REUSE_THRESHOLDS) || k_largest > REUSE_MAX_K)) ? 1u : 0u;
    const uint32_t tile_grid = (p.n_tiles + WAVES - 1) / WAVES;
    const uint32_t sub_grid = (p.n_tiles * SUB + WAVES - 1) / WAVES;
    const uint32_t light_grid = (p.n_tiles + LWAVES - 1) / LWAVES;
    const uint32_t scan_slices = (max_seg_tiles + SCAN_SLICE - 1) / SCAN_SLICE;

    const bool prof = (flags & GRAVAC_FLAG_PROFILE) != 0;
    if (prof && ns == 1)
        if (const int rc = refuse_capture(stream)) return rc;
    if (prof) {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        if (!g_ev_ready) {
            for (int i = 0; i < 4; ++i)
                if (hipEventCreate(&g_ev[i]) != hipSuccess) return GRAVAC_ERR_HIP;
            g_ev_ready = true;
        }
        (void)hipEventRecord(g_ev[0], stream);
    }
    static_assert(DENSE_ROUNDS == 4, "forms of the sampling kernel for 1, 2 and 4 groups per thread");
    if (p.have_sample) {
        hipLaunchKernelGGL(sample_rounds == 1 ? sample_kernel<1> : sample_rounds == 2 ? sample_kernel<2> : sample_kernel<4>,
                           dim3(p.n_sample_blocks), dim3(256), 0, stream, p);
    }
    hipLaunchKernelGGL(threshold_kernel, dim3(ns), dim3(1024), 0, stream, p);
    {
        // events 1 and 2 take the streaming kernel's own begin and end time stamps
        void (*kern)(Params) = single ? stream_kernel<SM_SINGLE, false>
                                      : (random ? stream_kernel<SM_EF, true> : stream_kernel<SM_EF, false>);
        if (prof)
            hipExtLaunchKernelGGL(kern, dim3(sub_grid), dim3(WG), 0, stream, g_ev[1], g_ev[2], 0, p);
        else
            hipLaunchKernelGGL(kern, dim3(sub_grid), dim3(WG), 0, stream, p);
    }
    hipLaunchKernelGGL(locate_kernel, dim3((uint32_t)(ns * n_cf)), dim3(256), 0, stream, p);
    // exact route, taken only by segments whose sampled bound failed (the kernels return at once otherwise)
    hipLaunchKernelGGL(coarse_kernel, dim3(tile_grid < XGRID ? tile_grid : XGRID), dim3(WG), 0, stream, p);
    if (random)
        hipLaunchKernelGGL((stream_kernel<SM_EXACT, true>), dim3(sub_grid < XGRID ? sub_grid : XGRID), dim3(WG), 0, stream, p);
    else
        hipLaunchKernelGGL((stream_kernel<SM_EXACT, false>), dim3(sub_grid < XGRID ? sub_grid : XGRID), dim3(WG), 0, stream, p);
    // exact resolution on the candidates, then count and emit
    // the candidate-list kernels with loops over the CFs exist for 1, 2, 4 and MAXCF CFs
    const int ncf_form = n_cf <= 1 ? 0 : n_cf <= 2 ? 1 : n_cf <= 4 ? 2 : 3;
    static_assert(MAXCF >= 4, "forms for 1, 2, 4 and MAXCF CFs");
    void (*const refine_forms[4])(Params) = {refine_kernel<1>, refine_kernel<2>, refine_kernel<4>, refine_kernel<MAXCF>};
    void (*const count_forms[4])(Params) = {count_kernel<1>, count_kernel<2>, count_kernel<4>, count_kernel<MAXCF>};
    hipLaunchKernelGGL(refine_forms[ncf_form], dim3(light_grid), dim3(LWG), 0, stream, p);
    hipLaunchKernelGGL(resolve_kernel, dim3(ns * n_cf), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(count_forms[ncf_form], dim3(light_grid), dim3(LWG), 0, stream, p);
    hipLaunchKernelGGL(scan_kernel, dim3(ns, scan_slices + n_cf), dim3(SCAN_T), 0, stream, p, scan_slices);
    hipLaunchKernelGGL(emit_kernel, dim3(light_grid), dim3(LWG), 0, stream, p);
    if (prof) {
        (void)hipEventRecord(g_ev[3], stream);
        g_ev_recorded = true;
    }
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
                         out_count, out_stats, workspace, workspace_bytes, flags, (hipStream_t)stream_v, nullptr, nullptr, 0, nullptr);
}

int gravac_randomk_compress(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                            uint64_t seed, const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val,
                            int64_t out_capacity, int64_t* out_count, double* out_stats, void* workspace,
                            size_t workspace_bytes, unsigned flags, void* stream_v)
{
    if (!residual) return GRAVAC_ERR_INVALID_ARG;
    return compress_impl(grad, residual, n, cf_list, n_cf, commit, seg_offsets, n_seg, out_idx, out_val, out_capacity,
                         out_count, out_stats, workspace, workspace_bytes, flags, (hipStream_t)stream_v, nullptr, nullptr, 0,
                         &seed);
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
                         idx1, residual, n, nullptr);
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
                           uint32_t* bounds, void* stream_v)
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
                               (const uint32_t*)bounds);
        } else {
            hipLaunchKernelGGL(decompress_kernel, dim3(grid), dim3(256), 0, stream, idx, val, wo, wn, n, dense_out);
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
    return decompress_impl(idx, val, counts, W, n, dense_out, (uint32_t*)workspace, stream_v);
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
    return decompress_impl(idx, val, counts, W, n, dense_out, bounds, stream_v);
}

int gravac_read_status(const void* workspace, void* stream_v, int32_t* out8)
{
    if (!workspace || !out8) return GRAVAC_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_v;
    if (hipStreamSynchronize(stream) != hipSuccess) return GRAVAC_ERR_HIP;
    Status s;
    if (hipMemcpy(&s, workspace, sizeof(Status), hipMemcpyDeviceToHost) != hipSuccess) return GRAVAC_ERR_HIP;
    out8[0] = s.any_fail; out8[1] = s.n_fail; out8[2] = s.error; out8[3] = s.n_seg; out8[4] = s.n_light;
    out8[5] = out8[6] = out8[7] = 0;
    return GRAVAC_OK;
}

int gravac_profile_read(float* stream_kernel_ms, float* total_ms)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_ev_ready || !g_ev_recorded) return GRAVAC_ERR_INVALID_ARG;
    if (hipEventSynchronize(g_ev[3]) != hipSuccess) return GRAVAC_ERR_HIP;
    float a = 0.f, b = 0.f;
    if (hipEventElapsedTime(&a, g_ev[1], g_ev[2]) != hipSuccess) return GRAVAC_ERR_HIP;
    if (hipEventElapsedTime(&b, g_ev[0], g_ev[3]) != hipSuccess) return GRAVAC_ERR_HIP;
    if (stream_kernel_ms) *stream_kernel_ms = a;
    if (total_ms) *total_ms = b;
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
