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
// resolve it to the exact key, count per tile, scan, emit the message in ascending index order
// and zero the selected residual slots.  If the sampled bound turns out wrong (fewer than k
// candidates, or a bin too coarse to resolve) the segment is redone by an exact route: a full
// 2048-bin histogram of the top key bits gives a bound that cannot fail.  Results are identical
// on both routes; only the number of passes over memory differs.
//
// Unit of work: a "wave tile" of TW consecutive elements handled by one 64-lane wavefront, which
// owns the slots [tile*TW, (tile+1)*TW) of the candidate arrays, so ordered compaction needs no
// communication between wavefronts and no tile can overflow.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <vector>

#include "gravac.h"

namespace {

constexpr int TW = 4096;            // elements per wave tile
constexpr int WG = 256;             // threads per workgroup of the tile kernels
constexpr int WAVES = WG / 64;
constexpr int ROW = 256;            // elements one wavefront touches per load (64 lanes x float4)
constexpr int NBIN = 2048;          // bins of the candidate / refine / coarse histograms
constexpr uint32_t OVF = NBIN - 1;  // last bin of the candidate histogram: everything above the bracket
constexpr int SBIN = 4096;          // bins of the sample histogram (key >> 19)
constexpr int SAMPLE_BLOCK = 1024;  // samples per workgroup of the sampling kernel
constexpr int SAMPLE_MAX = 65536;   // samples per segment at most (unless the segment is read whole)
constexpr int LCAP = 4096;          // keys a gather list can hold
constexpr int MAXCF = GRAVAC_MAX_CF;
constexpr double ZMARGIN = 5.0;     // safety margin of the sampled rank, in standard deviations

enum : uint32_t { MODE_RESOLVED = 0, MODE_GATHER = 1, MODE_HIST = 2, MODE_FAIL = 3 };

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
    uint32_t list_cnt;  // fill count of the gather list
    uint32_t pad[4];
};
static_assert(sizeof(CfState) == 64, "CfState layout");

struct SegState {
    uint32_t lo_min;  // smallest lo over the CFs: the candidate threshold of the segment
    uint32_t fail;    // 1 if the sampled bound failed and the segment takes the exact route
    uint32_t pad[2];
};

struct Status {
    int any_fail;
    int n_fail;
    int error;
    int n_seg;
    int pad[4];
};

typedef float v4f __attribute__((ext_vector_type(4)));

struct Params {
    const float* grad;
    float* res;
    int64_t n;
    int n_seg;  // >= 1
    int n_cf;
    int commit;
    unsigned flags;
    uint32_t n_tiles;
    uint32_t n_sample_blocks;
    // layerwise tables in the workspace (unused when n_seg == 1)
    const int64_t* seg_off;       // [n_seg + 1]
    const int64_t* koff;          // [n_seg + 1] output offset of each segment's message
    const uint32_t* tile_prefix;  // [n_seg + 1] first tile of each segment
    const uint32_t* samp_prefix;  // [n_seg + 1] first sample block of each segment
    const uint32_t* samp_cnt;     // [n_seg] samples of each segment
    const uint32_t* ktab;         // [n_seg][n_cf]
    // the same for one flat tensor
    uint32_t flat_k[MAXCF];
    uint32_t flat_samples;
    // workspace
    Status* status;
    CfState* st;     // [n_seg][n_cf]
    SegState* seg;   // [n_seg]
    uint32_t* hist1;     // [n_seg][n_cf][NBIN] candidate histogram
    uint32_t* hist2;     // [n_seg][n_cf][NBIN] refine histogram
    uint32_t* coarse;    // [n_seg][NBIN] histogram of key >> 20 (exact route)
    uint32_t* list;      // [n_seg][n_cf][LCAP] gather lists
    uint32_t* samp_key;  // [n_sample_blocks][SAMPLE_BLOCK]
    uint32_t* cand_cnt;  // [n_tiles]
    uint32_t* tg;        // [n_tiles] candidates with key > tau(commit)
    uint32_t* te;        // [n_tiles] candidates with key == tau(commit)
    uint32_t* toff;      // [n_tiles] offset of the tile's output inside its segment's message
    uint32_t* ttake;     // [n_tiles] how many of the tile's ties are selected
    double* ssd;         // [n_tiles] sum of acc^2
    double* sss;         // [n_tiles][n_cf] sum of acc^2 over keys > tau_j
    int32_t* cand_idx;   // [n_tiles][TW]
    float* cand_val;     // [n_tiles][TW]
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
__device__ __forceinline__ int64_t seg_begin(const Params& p, int t) { return is_flat(p) ? 0 : p.seg_off[t]; }
__device__ __forceinline__ int64_t seg_end(const Params& p, int t) { return is_flat(p) ? p.n : p.seg_off[t + 1]; }
__device__ __forceinline__ uint32_t seg_tile0(const Params& p, int t) { return is_flat(p) ? 0u : p.tile_prefix[t]; }
__device__ __forceinline__ uint32_t seg_tile1(const Params& p, int t) { return is_flat(p) ? p.n_tiles : p.tile_prefix[t + 1]; }
__device__ __forceinline__ uint32_t seg_k(const Params& p, int t, int j) { return is_flat(p) ? p.flat_k[j] : p.ktab[t * p.n_cf + j]; }
__device__ __forceinline__ int64_t seg_koff(const Params& p, int t) { return is_flat(p) ? 0 : p.koff[t]; }

// largest t with prefix[t] <= x, prefix ascending with prefix[0] == 0, n entries (excluding the end marker)
__device__ __forceinline__ int find_seg(const uint32_t* prefix, int n, uint32_t x)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (prefix[mid] <= x) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ int tile_seg(const Params& p, uint32_t u) { return is_flat(p) ? 0 : find_seg(p.tile_prefix, p.n_seg, u); }

__device__ __forceinline__ uint32_t key_of(float a) { return __float_as_uint(a) & 0x7FFFFFFFu; }

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

__device__ __forceinline__ uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// Inclusive suffix scan over the threads of a block (v of thread i becomes sum over i' >= i).
// tmp must hold blockDim.x entries.
__device__ __forceinline__ uint32_t block_suffix_scan(uint32_t v, uint32_t* tmp)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    tmp[tid] = v;
    __syncthreads();
    for (int o = 1; o < nt; o <<= 1) {
        uint32_t x = (tid + o < nt) ? tmp[tid + o] : 0u;
        __syncthreads();
        tmp[tid] += x;
        __syncthreads();
    }
    uint32_t r = tmp[tid];
    __syncthreads();
    return r;
}

// Inclusive prefix scan over the threads of a block.
__device__ __forceinline__ uint32_t block_prefix_scan(uint32_t v, uint32_t* tmp)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    tmp[tid] = v;
    __syncthreads();
    for (int o = 1; o < nt; o <<= 1) {
        uint32_t x = (tid >= o) ? tmp[tid - o] : 0u;
        __syncthreads();
        tmp[tid] += x;
        __syncthreads();
    }
    uint32_t r = tmp[tid];
    __syncthreads();
    return r;
}

// ---------------------------------------------------------------------------------------------
// K0a: sample acc = residual + grad at stratified positions, store the keys
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sample_kernel(Params p)
{
    const uint32_t b = blockIdx.x;
    const int t = is_flat(p) ? 0 : find_seg(p.samp_prefix, p.n_seg, b);
    const uint32_t lb = b - (is_flat(p) ? 0u : p.samp_prefix[t]);
    const uint32_t S = is_flat(p) ? p.flat_samples : p.samp_cnt[t];
    const int64_t s0 = seg_begin(p, t);
    const uint64_t nt = (uint64_t)(seg_end(p, t) - s0);
#pragma unroll
    for (int q = 0; q < SAMPLE_BLOCK / 256; ++q) {
        const uint32_t i = lb * SAMPLE_BLOCK + q * 256 + threadIdx.x;
        if (i < S) {
            uint64_t pos;
            if ((uint64_t)S == nt) {
                pos = i;  // the whole segment is read
            } else {
                const uint64_t a = ((uint64_t)i * nt) / S, e = ((uint64_t)(i + 1) * nt) / S;
                pos = a + hash32(i * 0x9E3779B9u + 0x85EBCA6Bu) % (uint32_t)(e - a);
            }
            const float acc = p.res[s0 + (int64_t)pos] + p.grad[s0 + (int64_t)pos];
            p.samp_key[(size_t)b * SAMPLE_BLOCK + q * 256 + threadIdx.x] = key_of(acc);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// K0b: per segment, turn the sampled keys into (lo, s) per CF; clear the segment's histograms
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void threshold_kernel(Params p)
{
    __shared__ uint32_t hist[SBIN];
    __shared__ uint32_t tmp[1024];
    __shared__ uint32_t found[2];
    const int t = blockIdx.x, tid = threadIdx.x;
    const uint32_t S = is_flat(p) ? p.flat_samples : p.samp_cnt[t];
    const uint32_t sb0 = is_flat(p) ? 0u : p.samp_prefix[t];
    const uint64_t nt = (uint64_t)(seg_end(p, t) - seg_begin(p, t));
    const bool whole = ((uint64_t)S == nt);

    for (int i = tid; i < SBIN; i += 1024) hist[i] = 0;
    for (int i = tid; i < p.n_cf * NBIN; i += 1024) p.hist1[(size_t)t * p.n_cf * NBIN + i] = 0;
    for (int i = tid; i < NBIN; i += 1024) p.coarse[(size_t)t * NBIN + i] = 0;
    if (t == 0 && tid == 0) {
        p.status->any_fail = 0; p.status->n_fail = 0; p.status->error = 0; p.status->n_seg = p.n_seg;
    }
    __syncthreads();
    const bool forced = (p.flags & GRAVAC_FLAG_FORCE_FALLBACK) != 0;
    if (!forced)
        for (uint32_t i = tid; i < S; i += 1024) atomicAdd(&hist[p.samp_key[(size_t)sb0 * SAMPLE_BLOCK + i] >> 19], 1u);
    __syncthreads();
    // thread i owns bins 4i .. 4i+3
    const uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
    const uint32_t mine = h0 + h1 + h2 + h3;
    const uint32_t suf = block_suffix_scan(mine, tmp);  // samples in bins >= 4*tid

    uint32_t lo_min = 0xFFFFFFFFu;
    for (int j = 0; j < p.n_cf; ++j) {
        const uint32_t k = seg_k(p, t, j);
        uint32_t r_lo, r_hi;
        if (whole) {
            r_lo = r_hi = k;
        } else {
            const double m = (double)k * (double)S / (double)nt, sd = sqrt(m);
            const double a = ceil(m + ZMARGIN * sd + 2.0), b = floor(m - ZMARGIN * sd - 2.0);
            r_lo = (a >= 4.0e9) ? 0xFFFFFFFFu : (uint32_t)a;
            r_hi = (b < 1.0) ? 1u : (uint32_t)b;
        }
        if (tid == 0) { found[0] = 0; found[1] = SBIN - 1; }
        __syncthreads();
        // bin of the r-th largest sample: above < r <= above + count
        uint32_t above = suf - mine;
        const uint32_t hh[4] = {h0, h1, h2, h3};
#pragma unroll
        for (int q = 3; q >= 0; --q) {
            const uint32_t c = hh[q];
            if (above < r_lo && above + c >= r_lo) found[0] = 4 * tid + q;
            if (above < r_hi && above + c >= r_hi) found[1] = 4 * tid + q;
            above += c;
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t lo = found[0] << 19;                 // lower edge; bin 0 if the sample has < r_lo keys
            const uint64_t hi = ((uint64_t)found[1] + 1) << 19;  // upper edge of the bin of the r_hi-th
            uint32_t s = 0;
            while ((((hi > lo ? hi - lo : 0)) >> s) > (uint64_t)OVF) ++s;
            if (forced) { lo = 0xFFFFFFFFu; s = 0; }
            CfState st;
            st.k = k; st.lo = lo; st.s = s; st.mode = MODE_FAIL; st.base = 0; st.open = 0; st.above = 0; st.c = 0;
            st.tau = 0; st.need = 0; st.cnt_gt = 0; st.list_cnt = 0;
            st.pad[0] = st.pad[1] = st.pad[2] = st.pad[3] = 0;
            p.st[(size_t)t * p.n_cf + j] = st;
            lo_min = lo < lo_min ? lo : lo_min;
        }
        __syncthreads();
    }
    if (tid == 0) {
        SegState ss;
        ss.lo_min = lo_min; ss.fail = 0; ss.pad[0] = ss.pad[1] = 0;
        p.seg[t] = ss;
    }
}

// ---------------------------------------------------------------------------------------------
// K1: the streaming pass.  EF = true: read grad and residual, write acc back, sum acc^2.
//     EF = false (exact route): read acc from residual only.  Both collect candidates.
// ---------------------------------------------------------------------------------------------
struct TileCtx {
    uint32_t lo_min;
    uint32_t lo[MAXCF];
    uint32_t sh[MAXCF];
    uint32_t ovf[MAXCF];
    uint32_t* h1;       // candidate histograms of this tile's segment
    int32_t* cidx;      // candidate slots of this tile
    float* cval;
    uint32_t run;       // candidates written so far
    double ssd;
    int ncf;
};

__device__ __forceinline__ void cand_hist(TileCtx& c, uint32_t key)
{
#pragma unroll
    for (int j = 0; j < MAXCF; ++j) {
        if (j < c.ncf && key >= c.lo[j]) {
            const uint32_t b = (key - c.lo[j]) >> c.sh[j];
            if (b >= OVF) c.ovf[j]++;
            else atomicAdd(&c.h1[j * NBIN + b], 1u);
        }
    }
}

// One lane's four consecutive elements a[0..3] at global index g, vm = validity bits.
template <bool EF>
__device__ __forceinline__ void consume(TileCtx& c, const float a[4], int64_t g, unsigned vm)
{
    uint32_t key[4];
    bool f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        key[e] = key_of(a[e]);
        const bool valid = (vm >> e) & 1u;
        f[e] = valid && key[e] >= c.lo_min;
        if (EF) {
            const double d = valid ? (double)a[e] : 0.0;
            c.ssd += d * d;
        }
    }
    const bool any = f[0] | f[1] | f[2] | f[3];
    if (__ballot(any) != 0ull) {
        uint64_t m[4];
        uint32_t pre = 0, tot = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            m[e] = __ballot(f[e]);
            pre += lanes_below(m[e]);
            tot += (uint32_t)__popcll(m[e]);
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

template <bool EF>
__global__ __launch_bounds__(WG) void stream_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * WAVES;
    if (!EF && p.status->any_fail == 0) return;

    for (uint32_t u = wave; u < p.n_tiles; u += nwaves) {
        const int t = tile_seg(p, u);
        if (!EF && p.seg[t].fail == 0) continue;
        const int64_t sb = seg_begin(p, t), se = seg_end(p, t);
        const int64_t s0 = sb + (int64_t)(u - seg_tile0(p, t)) * TW;
        const int64_t e0 = (s0 + TW < se) ? s0 + TW : se;

        TileCtx c;
        c.ncf = p.n_cf;
        c.lo_min = p.seg[t].lo_min;
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) {
            c.ovf[j] = 0;
            if (j < p.n_cf) {
                c.lo[j] = p.st[(size_t)t * p.n_cf + j].lo;
                c.sh[j] = p.st[(size_t)t * p.n_cf + j].s;
            } else {
                c.lo[j] = 0xFFFFFFFFu;
                c.sh[j] = 0;
            }
        }
        c.h1 = p.hist1 + (size_t)t * p.n_cf * NBIN;
        c.cidx = p.cand_idx + (size_t)u * TW;
        c.cval = p.cand_val + (size_t)u * TW;
        c.run = 0;
        c.ssd = 0.0;

        int64_t rb = s0 & ~(int64_t)3;  // rows start at a multiple of 4 elements (16-byte aligned vectors)
        // head row(s) until the row lies fully inside the tile
        for (; rb < e0; rb += ROW) {
            const bool full = (rb >= s0) && (rb + ROW <= e0);
            if (full) {
                // four full rows at a time: all loads first, then the arithmetic
                if (rb + 4 * ROW <= e0) {
                    v4f gv[4], rv[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int64_t g = rb + q * ROW + 4 * lane;
                        rv[q] = __builtin_nontemporal_load((const v4f*)(p.res + g));
                        if (EF) gv[q] = __builtin_nontemporal_load((const v4f*)(p.grad + g));
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int64_t g = rb + q * ROW + 4 * lane;
                        float a[4];
                        if (EF) {
                            const v4f av = rv[q] + gv[q];
                            __builtin_nontemporal_store(av, (v4f*)(p.res + g));
                            a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
                        } else {
                            a[0] = rv[q].x; a[1] = rv[q].y; a[2] = rv[q].z; a[3] = rv[q].w;
                        }
                        consume<EF>(c, a, g, 0xFu);
                    }
                    rb += 3 * ROW;
                    continue;
                }
                const int64_t g = rb + 4 * lane;
                v4f rv = __builtin_nontemporal_load((const v4f*)(p.res + g));
                float a[4];
                if (EF) {
                    const v4f gv = __builtin_nontemporal_load((const v4f*)(p.grad + g));
                    const v4f av = rv + gv;
                    __builtin_nontemporal_store(av, (v4f*)(p.res + g));
                    a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
                } else {
                    a[0] = rv.x; a[1] = rv.y; a[2] = rv.z; a[3] = rv.w;
                }
                consume<EF>(c, a, g, 0xFu);
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
                        if (EF) {
                            a[e] = p.res[q] + p.grad[q];
                            p.res[q] = a[e];
                        } else {
                            a[e] = p.res[q];
                        }
                    }
                }
                consume<EF>(c, a, g, vm);
            }
        }

        // tile epilogue
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) {
            if (j < p.n_cf) {
                const uint32_t o = wave_sum(c.ovf[j]);
                if (lane == 0 && o) atomicAdd(&c.h1[j * NBIN + OVF], o);
            }
        }
        if (EF) {
            const double s = wave_sum(c.ssd);
            if (lane == 0) p.ssd[u] = s;
        }
        if (lane == 0) p.cand_cnt[u] = c.run;
    }
}

// ---------------------------------------------------------------------------------------------
// F1 (exact route): histogram of key >> 20 over the tiles of failed segments
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void coarse_kernel(Params p)
{
    __shared__ uint32_t lh[WAVES][NBIN];
    if (p.status->any_fail == 0) return;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + wib);
    const uint32_t nwaves = gridDim.x * WAVES;
    uint32_t* h = lh[wib];
    for (uint32_t u = wave; u < p.n_tiles; u += nwaves) {
        const int t = tile_seg(p, u);
        if (p.seg[t].fail == 0) continue;
        const int64_t sb = seg_begin(p, t), se = seg_end(p, t);
        const int64_t s0 = sb + (int64_t)(u - seg_tile0(p, t)) * TW;
        const int64_t e0 = (s0 + TW < se) ? s0 + TW : se;
        for (int i = lane; i < NBIN; i += 64) h[i] = 0;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
        for (int64_t q = s0 + lane; q < e0; q += 64) atomicAdd(&h[key_of(p.res[q]) >> 20], 1u);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
        uint32_t* gh = p.coarse + (size_t)t * NBIN;
        for (int i = lane; i < NBIN; i += 64) {
            const uint32_t v = h[i];
            if (v) atomicAdd(&gh[i], v);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    }
}

// Find the bin that holds the k-th largest: scanning from the top bin down,
// above < k <= above + count.  One block of 256 threads, thread i owns bins 8i .. 8i+7.
// Returns through out[0..2] = {bin, above, count}; out[3] = total.  Call with all threads.
__device__ __forceinline__ void locate_bin(const uint32_t* hist, uint32_t k, uint32_t* tmp, uint32_t* out)
{
    const int tid = threadIdx.x;
    uint32_t h[8], mine = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) { h[q] = hist[8 * tid + q]; mine += h[q]; }
    const uint32_t suf = block_suffix_scan(mine, tmp);
    if (tid == 0) { out[0] = 0xFFFFFFFFu; out[1] = 0; out[2] = 0; out[3] = suf; }
    __syncthreads();
    uint32_t above = suf - mine;
#pragma unroll
    for (int q = 7; q >= 0; --q) {
        if (above < k && above + h[q] >= k) { out[0] = 8 * tid + q; out[1] = above; out[2] = h[q]; }
        above += h[q];
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// LC (exact route): per (failed segment, CF) set lo to the base of the coarse bin of the k-th largest
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void locate_coarse_kernel(Params p)
{
    __shared__ uint32_t tmp[256];
    __shared__ uint32_t out[4];
    if (p.status->any_fail == 0) return;
    const int t = blockIdx.x, j = blockIdx.y, tid = threadIdx.x;
    if (p.seg[t].fail == 0) return;
    CfState* st = &p.st[(size_t)t * p.n_cf + j];
    const uint32_t k = st->k;
    locate_bin(p.coarse + (size_t)t * NBIN, k, tmp, out);
    for (int i = tid; i < NBIN; i += 256) p.hist1[((size_t)t * p.n_cf + j) * NBIN + i] = 0;
    if (tid == 0) {
        if (out[0] == 0xFFFFFFFFu) { p.status->error = 1; out[0] = 0; }
        const uint32_t lo = out[0] << 20;
        st->lo = lo;
        st->s = 10;  // 1024 bins of 2^10 keys cover the coarse bin; keys above it land in the open last bin
        st->mode = MODE_FAIL; st->list_cnt = 0;
        atomicMin(&p.seg[t].lo_min, lo);
    }
}

// ---------------------------------------------------------------------------------------------
// L1: per (segment, CF) find the candidate-histogram bin of the k-th largest and decide how to resolve it
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void locate_kernel(Params p, int second)
{
    __shared__ uint32_t tmp[256];
    __shared__ uint32_t out[4];
    const int t = blockIdx.x, j = blockIdx.y, tid = threadIdx.x;
    if (second) {
        if (p.status->any_fail == 0) return;
        if (p.seg[t].fail == 0) return;
    }
    CfState* st = &p.st[(size_t)t * p.n_cf + j];
    const uint32_t k = st->k, lo = st->lo, s = st->s;
    locate_bin(p.hist1 + ((size_t)t * p.n_cf + j) * NBIN, k, tmp, out);
    const uint32_t b = out[0], above = out[1], c = out[2];
    uint32_t mode;
    if (b == 0xFFFFFFFFu) {
        mode = MODE_FAIL;  // fewer than k candidates: the bound was too high
    } else if (b == OVF) {
        mode = (c <= LCAP) ? MODE_GATHER : MODE_FAIL;
    } else if (s == 0) {
        mode = MODE_RESOLVED;
    } else if (c <= LCAP) {
        mode = MODE_GATHER;
    } else if (s <= 11) {
        mode = MODE_HIST;
    } else {
        mode = MODE_FAIL;
    }
    if (mode == MODE_HIST)
        for (int i = tid; i < NBIN; i += 256) p.hist2[((size_t)t * p.n_cf + j) * NBIN + i] = 0;
    if (tid == 0) {
        st->mode = mode;
        st->list_cnt = 0;
        if (mode != MODE_FAIL) {
            st->base = lo + (b << s);
            st->open = (b == OVF) ? 1u : 0u;
            st->above = above;
            st->c = c;
            if (mode == MODE_RESOLVED) { st->tau = st->base; st->cnt_gt = above; st->need = k - above; }
        } else if (second) {
            p.status->error = 1;
        } else {
            p.status->any_fail = 1;
            if (atomicExch(&p.seg[t].fail, 1u) == 0u) atomicAdd(&p.status->n_fail, 1);
            p.seg[t].lo_min = 0xFFFFFFFFu;  // the exact route lowers it again with atomicMin
        }
    }
}

// ---------------------------------------------------------------------------------------------
// R1: one pass over the candidates: gather (or histogram) the keys of the bin that holds the k-th largest
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void refine_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * WAVES;
    for (uint32_t u = wave; u < p.n_tiles; u += nwaves) {
        const uint32_t cnt = p.cand_cnt[u];
        if (cnt == 0) continue;
        const int t = tile_seg(p, u);
        uint32_t mode[MAXCF], base[MAXCF], span[MAXCF];
        bool work = false;
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) {
            mode[j] = MODE_RESOLVED; base[j] = 0; span[j] = 0;
            if (j < p.n_cf) {
                const CfState* st = &p.st[(size_t)t * p.n_cf + j];
                mode[j] = st->mode;
                base[j] = st->base;
                span[j] = st->open ? 0xFFFFFFFFu : ((1u << st->s) - 1u);  // key - base <= span
                work |= (mode[j] == MODE_GATHER || mode[j] == MODE_HIST);
            }
        }
        if (!work) continue;
        const float* cv = p.cand_val + (size_t)u * TW;
        for (uint32_t i = lane; i < cnt; i += 64) {
            const uint32_t key = key_of(cv[i]);
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) {
                if (j < p.n_cf && key >= base[j] && key - base[j] <= span[j]) {
                    CfState* st = &p.st[(size_t)t * p.n_cf + j];
                    if (mode[j] == MODE_GATHER) {
                        const uint32_t pos = atomicAdd(&st->list_cnt, 1u);
                        if (pos < LCAP) p.list[((size_t)t * p.n_cf + j) * LCAP + pos] = key;
                    } else if (mode[j] == MODE_HIST) {
                        atomicAdd(&p.hist2[((size_t)t * p.n_cf + j) * NBIN + (key - base[j])], 1u);
                    }
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
    __shared__ uint32_t tmp[256];
    __shared__ uint32_t out[4];
    __shared__ uint32_t keys[LCAP];
    __shared__ uint32_t wsum[WAVES];
    const int t = blockIdx.x, j = blockIdx.y, tid = threadIdx.x;
    CfState* st = &p.st[(size_t)t * p.n_cf + j];
    const uint32_t mode = st->mode;
    if (mode == MODE_RESOLVED) return;
    if (mode == MODE_FAIL) { if (tid == 0) p.status->error = 1; return; }
    const uint32_t k = st->k, above = st->above, want = k - above;  // want-th largest inside the bin
    if (mode == MODE_HIST) {
        // bins are single keys: base + b
        locate_bin(p.hist2 + ((size_t)t * p.n_cf + j) * NBIN, want, tmp, out);
        if (tid == 0) {
            if (out[0] == 0xFFFFFFFFu) { p.status->error = 1; out[0] = 0; }
            st->tau = st->base + out[0];
            st->cnt_gt = above + out[1];
            st->need = k - st->cnt_gt;
            st->mode = MODE_RESOLVED;
        }
        return;
    }
    // gather: the want-th largest of the listed keys by a bitwise search on the key value
    const uint32_t c = st->c;
    if (st->list_cnt != c || c > LCAP || want == 0 || want > c) { if (tid == 0) p.status->error = 1; return; }
    const uint32_t* lst = p.list + ((size_t)t * p.n_cf + j) * LCAP;
    for (uint32_t i = tid; i < c; i += 256) keys[i] = lst[i];
    __syncthreads();
    uint32_t prefix = 0;
    for (int bit = 30; bit >= 0; --bit) {
        const uint32_t trial = prefix | (1u << bit);
        uint32_t cnt = 0;
        for (uint32_t i = tid; i < c; i += 256) cnt += (keys[i] >= trial);
        cnt = wave_sum(cnt);
        if ((tid & 63) == 0) wsum[tid >> 6] = cnt;
        __syncthreads();
        const uint32_t total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
        __syncthreads();
        if (total >= want) prefix = trial;
    }
    uint32_t gt = 0;
    for (uint32_t i = tid; i < c; i += 256) gt += (keys[i] > prefix);
    gt = wave_sum(gt);
    if ((tid & 63) == 0) wsum[tid >> 6] = gt;
    __syncthreads();
    if (tid == 0) {
        st->tau = prefix;
        st->cnt_gt = above + wsum[0] + wsum[1] + wsum[2] + wsum[3];
        st->need = k - st->cnt_gt;
        st->mode = MODE_RESOLVED;
    }
}

// ---------------------------------------------------------------------------------------------
// K3: per tile, count candidates above / at the committed threshold; energy above each CF's threshold
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void tile_count_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * WAVES;
    for (uint32_t u = wave; u < p.n_tiles; u += nwaves) {
        const uint32_t cnt = p.cand_cnt[u];
        uint32_t g = 0, e = 0;
        double ss[MAXCF];
#pragma unroll
        for (int j = 0; j < MAXCF; ++j) ss[j] = 0.0;
        if (cnt) {
            const int t = tile_seg(p, u);
            uint32_t tau[MAXCF];
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) tau[j] = (j < p.n_cf) ? p.st[(size_t)t * p.n_cf + j].tau : 0xFFFFFFFFu;
            uint32_t tc = 0;
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) if (j == p.commit) tc = tau[j];
            const float* cv = p.cand_val + (size_t)u * TW;
            for (uint32_t i = lane; i < cnt; i += 64) {
                const float v = cv[i];
                const uint32_t key = key_of(v);
                const double d = (double)v;
                g += (key > tc);
                e += (key == tc);
#pragma unroll
                for (int j = 0; j < MAXCF; ++j) if (j < p.n_cf && key > tau[j]) ss[j] += d * d;
            }
            g = wave_sum(g);
            e = wave_sum(e);
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) if (j < p.n_cf) ss[j] = wave_sum(ss[j]);
        }
        if (lane == 0) {
            p.tg[u] = g;
            p.te[u] = e;
#pragma unroll
            for (int j = 0; j < MAXCF; ++j) if (j < p.n_cf) p.sss[(size_t)u * p.n_cf + j] = ss[j];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// SCAN: blockIdx.y == 0: per segment exclusive scan of the tile counts -> output offsets and tie quotas.
//       blockIdx.y == 1 + j: statistics of CF j (fixed summation order).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void scan_kernel(Params p)
{
    __shared__ uint32_t tmp[1024];
    __shared__ double dsum[2][1024];
    const int t = blockIdx.x, role = blockIdx.y, tid = threadIdx.x, nt = blockDim.x;
    const uint32_t u0 = seg_tile0(p, t), u1 = seg_tile1(p, t), ntile = u1 - u0;
    if (role == 0) {
        const uint32_t need = p.st[(size_t)t * p.n_cf + p.commit].need;
        const uint32_t chunk = (ntile + nt - 1) / nt;
        const uint32_t a = u0 + tid * chunk < u1 ? u0 + tid * chunk : u1;
        const uint32_t b = a + chunk < u1 ? a + chunk : u1;
        uint32_t G = 0, E = 0;
        for (uint32_t u = a; u < b; ++u) { G += p.tg[u]; E += p.te[u]; }
        uint32_t Gx = block_prefix_scan(G, tmp) - G;
        uint32_t Ex = block_prefix_scan(E, tmp) - E;
        for (uint32_t u = a; u < b; ++u) {
            const uint32_t g = p.tg[u], e = p.te[u];
            const uint32_t ties_before = Ex < need ? Ex : need;
            const uint32_t left = need - ties_before;
            p.toff[u] = Gx + ties_before;
            p.ttake[u] = left < e ? left : e;
            Gx += g;
            Ex += e;
        }
        if (t == 0 && tid == 0 && p.out_count) {
            int64_t total = 0;
            if (is_flat(p)) total = p.flat_k[p.commit]; else total = p.koff[p.n_seg];
            *p.out_count = total;
        }
        return;
    }
    const int j = role - 1;
    double sd = 0.0, sj = 0.0;
    for (uint32_t u = u0 + tid; u < u1; u += nt) {
        sd += p.ssd[u];
        sj += p.sss[(size_t)u * p.n_cf + j];
    }
    dsum[0][tid] = sd;
    dsum[1][tid] = sj;
    __syncthreads();
    for (int o = nt >> 1; o > 0; o >>= 1) {
        if (tid < o) { dsum[0][tid] += dsum[0][tid + o]; dsum[1][tid] += dsum[1][tid + o]; }
        __syncthreads();
    }
    if (tid == 0) {
        const CfState* st = &p.st[(size_t)t * p.n_cf + j];
        const double tau = (double)__uint_as_float(st->tau);
        const double ss_dense = dsum[0][0];
        const double ss_sel = dsum[1][0] + (double)st->need * tau * tau;
        double* o = p.out_stats + ((size_t)t * p.n_cf + j) * GRAVAC_STATS_PER_CF;
        o[0] = ss_sel;
        o[1] = ss_dense;
        o[2] = (ss_dense == 0.0) ? 1.0 : ss_sel / ss_dense;
        o[3] = tau;
    }
}

// ---------------------------------------------------------------------------------------------
// K4: emit the committed selection in ascending index order and zero its residual slots
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void emit_kernel(Params p)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(blockIdx.x * WAVES + (threadIdx.x >> 6));
    const uint32_t nwaves = gridDim.x * WAVES;
    for (uint32_t u = wave; u < p.n_tiles; u += nwaves) {
        const uint32_t cnt = p.cand_cnt[u];
        if (cnt == 0) continue;
        const uint32_t take = p.ttake[u];
        if (p.tg[u] == 0 && take == 0) continue;
        const int t = tile_seg(p, u);
        const uint32_t tau = p.st[(size_t)t * p.n_cf + p.commit].tau;
        int64_t pos = seg_koff(p, t) + (int64_t)p.toff[u];
        const int64_t lim = seg_koff(p, t) + (int64_t)seg_k(p, t, p.commit);  // end of this segment's message
        uint32_t erun = 0;
        const float* cv = p.cand_val + (size_t)u * TW;
        const int32_t* ci = p.cand_idx + (size_t)u * TW;
        for (uint32_t i0 = 0; i0 < cnt; i0 += 64) {
            const uint32_t i = i0 + lane;
            float v = 0.0f;
            int32_t ix = 0;
            bool gt = false, eq = false;
            if (i < cnt) {
                v = cv[i];
                ix = ci[i];
                const uint32_t key = key_of(v);
                gt = key > tau;
                eq = key == tau;
            }
            const uint64_t me = __ballot(eq);
            const bool sel = gt || (eq && (erun + lanes_below(me)) < take);
            const uint64_t ms = __ballot(sel);
            if (sel) {
                const int64_t o = pos + lanes_below(ms);
                if (o < lim) {
                    p.out_idx[o] = ix;
                    p.out_val[o] = v;
                    p.res[ix] = 0.0f;
                } else {
                    p.status->error = 1;  // cannot happen if the counts are consistent; never write out of range
                }
            }
            pos += __popcll(ms);
            erun += (uint32_t)__popcll(me);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// decompression: dense_out[idx] += val, workers in order, one workgroup per tile of dense_out
// ---------------------------------------------------------------------------------------------
constexpr int DTILE = 8192;  // floats of dense_out per workgroup (32 KiB of LDS)
constexpr int DMAXW = 64;    // workers per launch

struct WorkerOffsets {
    int64_t at[DMAXW + 1];
};

__device__ __forceinline__ int64_t lower_bound_i32(const int32_t* a, int64_t lo, int64_t hi, int64_t x)
{
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if ((int64_t)a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(256) void decompress_kernel(const int32_t* __restrict__ idx, const float* __restrict__ val,
                                                         WorkerOffsets wo, int W, int64_t n, float* dense)
{
    __shared__ float acc[DTILE];
    __shared__ int64_t lo[DMAXW], hi[DMAXW];
    __shared__ int any;
    const int tid = threadIdx.x;
    const bool vec = (((uintptr_t)dense) & 15) == 0;  // float4 access needs a 16-byte aligned buffer
    const int64_t ntile = (n + DTILE - 1) / DTILE;
    for (int64_t tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        const int64_t base = tile * DTILE;
        const int len = (int)((n - base < DTILE) ? n - base : DTILE);
        if (tid == 0) any = 0;
        __syncthreads();
        if (tid < 2 * W) {
            const int w = tid >> 1;
            const int64_t x = (tid & 1) ? base + len : base;
            const int64_t r = lower_bound_i32(idx, wo.at[w], wo.at[w + 1], x);
            if (tid & 1) hi[w] = r; else lo[w] = r;
        }
        __syncthreads();
        if (tid < W && hi[tid] > lo[tid]) any = 1;
        __syncthreads();
        if (any) {
            for (int i = tid * 4; i < len; i += 256 * 4) {
                if (vec && i + 4 <= len) {
                    const v4f v = *(const v4f*)(dense + base + i);
                    acc[i] = v.x; acc[i + 1] = v.y; acc[i + 2] = v.z; acc[i + 3] = v.w;
                } else {
                    for (int e = 0; e < 4 && i + e < len; ++e) acc[i + e] = dense[base + i + e];
                }
            }
            __syncthreads();
            for (int w = 0; w < W; ++w) {
                for (int64_t q = lo[w] + tid; q < hi[w]; q += 256) {
                    const int64_t j = (int64_t)idx[q] - base;
                    if (j >= 0 && j < len) acc[j] += val[q];
                }
                __syncthreads();
            }
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
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t status, seg_off, koff, tile_prefix, samp_prefix, samp_cnt, ktab, st, seg, hist1, hist2, coarse, list,
        samp_key, cand_cnt, tg, te, toff, ttake, ssd, sss, cand_idx, cand_val, total;
};

// Upper bounds that depend only on (n, n_cf, n_seg).
uint64_t max_tiles(int64_t n, int n_seg) { return (uint64_t)((n + TW - 1) / TW) + (uint64_t)n_seg; }

uint64_t max_sample_blocks(int64_t n, int n_seg)
{
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
    L.seg_off = take(sizeof(int64_t) * (n_seg + 1));
    L.koff = take(sizeof(int64_t) * (n_seg + 1));
    L.tile_prefix = take(sizeof(uint32_t) * (n_seg + 1));
    L.samp_prefix = take(sizeof(uint32_t) * (n_seg + 1));
    L.samp_cnt = take(sizeof(uint32_t) * n_seg);
    L.ktab = take(sizeof(uint32_t) * sc);
    L.st = take(sizeof(CfState) * sc);
    L.seg = take(sizeof(SegState) * n_seg);
    L.hist1 = take(sizeof(uint32_t) * sc * NBIN);
    L.hist2 = take(sizeof(uint32_t) * sc * NBIN);
    L.coarse = take(sizeof(uint32_t) * (size_t)n_seg * NBIN);
    L.list = take(sizeof(uint32_t) * sc * LCAP);
    L.samp_key = take(sizeof(uint32_t) * nsb * SAMPLE_BLOCK);
    L.cand_cnt = take(sizeof(uint32_t) * nt);
    L.tg = take(sizeof(uint32_t) * nt);
    L.te = take(sizeof(uint32_t) * nt);
    L.toff = take(sizeof(uint32_t) * nt);
    L.ttake = take(sizeof(uint32_t) * nt);
    L.ssd = take(sizeof(double) * nt);
    L.sss = take(sizeof(double) * nt * n_cf);
    L.cand_idx = take(sizeof(int32_t) * nt * TW);
    L.cand_val = take(sizeof(float) * nt * TW);
    L.total = at;
    return L;
}

// samples taken from a segment of nt elements when the largest CF is cf_max
uint32_t sample_count(uint64_t nt, double cf_max, bool flat)
{
    uint64_t target = flat ? (uint64_t)SAMPLE_MAX : (uint64_t)(32.0 * std::ceil(cf_max));
    if (target < 4096) target = 4096;
    if (target > (uint64_t)SAMPLE_MAX) target = SAMPLE_MAX;
    target = (target + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK * SAMPLE_BLOCK;
    return (nt <= 2 * target) ? (uint32_t)nt : (uint32_t)target;
}

int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

std::mutex g_prof_mutex;
hipEvent_t g_ev[4];
bool g_ev_ready = false;
bool g_ev_recorded = false;

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

int gravac_compress(const float* grad, float* residual, int64_t n, const double* cf_list, int n_cf, int commit,
                    const int64_t* seg_offsets, int n_seg, int32_t* out_idx, float* out_val, int64_t out_capacity,
                    int64_t* out_count, double* out_stats, void* workspace, size_t workspace_bytes, unsigned flags,
                    void* stream_v)
{
    hipStream_t stream = (hipStream_t)stream_v;
    if (!grad || !residual || !cf_list || !out_idx || !out_val || !out_stats) return GRAVAC_ERR_INVALID_ARG;
    if (n <= 0 || n > 2147483647LL || n_cf < 1 || n_cf > MAXCF || commit < 0 || commit >= n_cf) return GRAVAC_ERR_INVALID_ARG;
    if (((uintptr_t)grad & 15) || ((uintptr_t)residual & 15)) return GRAVAC_ERR_INVALID_ARG;
    if (n_seg < 0 || (n_seg > 0 && !seg_offsets) || (int64_t)n_seg > n) return GRAVAC_ERR_INVALID_ARG;
    double cf_max = 1.0;
    for (int j = 0; j < n_cf; ++j) {
        if (!(cf_list[j] >= 1.0) || std::isinf(cf_list[j])) return GRAVAC_ERR_INVALID_ARG;
        if (cf_list[j] > cf_max) cf_max = cf_list[j];
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
    p.grad = grad; p.res = residual; p.n = n; p.n_seg = ns; p.n_cf = n_cf; p.commit = commit; p.flags = flags;
    p.status = (Status*)(ws + L.status);
    p.seg_off = (const int64_t*)(ws + L.seg_off);
    p.koff = (const int64_t*)(ws + L.koff);
    p.tile_prefix = (const uint32_t*)(ws + L.tile_prefix);
    p.samp_prefix = (const uint32_t*)(ws + L.samp_prefix);
    p.samp_cnt = (const uint32_t*)(ws + L.samp_cnt);
    p.ktab = (const uint32_t*)(ws + L.ktab);
    p.st = (CfState*)(ws + L.st);
    p.seg = (SegState*)(ws + L.seg);
    p.hist1 = (uint32_t*)(ws + L.hist1);
    p.hist2 = (uint32_t*)(ws + L.hist2);
    p.coarse = (uint32_t*)(ws + L.coarse);
    p.list = (uint32_t*)(ws + L.list);
    p.samp_key = (uint32_t*)(ws + L.samp_key);
    p.cand_cnt = (uint32_t*)(ws + L.cand_cnt);
    p.tg = (uint32_t*)(ws + L.tg);
    p.te = (uint32_t*)(ws + L.te);
    p.toff = (uint32_t*)(ws + L.toff);
    p.ttake = (uint32_t*)(ws + L.ttake);
    p.ssd = (double*)(ws + L.ssd);
    p.sss = (double*)(ws + L.sss);
    p.cand_idx = (int32_t*)(ws + L.cand_idx);
    p.cand_val = (float*)(ws + L.cand_val);
    p.out_idx = out_idx; p.out_val = out_val; p.out_count = out_count; p.out_stats = out_stats;

    int64_t total_out = 0;
    if (ns == 1) {
        for (int j = 0; j < n_cf; ++j) p.flat_k[j] = (uint32_t)gravac_topk_count(n, cf_list[j]);
        p.flat_samples = sample_count((uint64_t)n, cf_max, true);
        p.n_tiles = (uint32_t)((n + TW - 1) / TW);
        p.n_sample_blocks = (p.flat_samples + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
        total_out = p.flat_k[commit];
        if (total_out > out_capacity) return GRAVAC_ERR_CAPACITY;
    } else {
        // layerwise tables, built on the host and copied into the workspace in one piece
        std::vector<int64_t> koff(ns + 1);
        std::vector<uint32_t> tile_prefix(ns + 1), samp_prefix(ns + 1), samp_cnt(ns), ktab((size_t)ns * n_cf);
        uint64_t tiles = 0, sblocks = 0;
        for (int t = 0; t < ns; ++t) {
            const int64_t nt = seg_offsets[t + 1] - seg_offsets[t];
            koff[t] = total_out;
            tile_prefix[t] = (uint32_t)tiles;
            samp_prefix[t] = (uint32_t)sblocks;
            for (int j = 0; j < n_cf; ++j) ktab[(size_t)t * n_cf + j] = (uint32_t)gravac_topk_count(nt, cf_list[j]);
            total_out += ktab[(size_t)t * n_cf + commit];
            samp_cnt[t] = sample_count((uint64_t)nt, cf_max, false);
            tiles += (uint64_t)((nt + TW - 1) / TW);
            sblocks += (samp_cnt[t] + SAMPLE_BLOCK - 1) / SAMPLE_BLOCK;
        }
        koff[ns] = total_out;
        tile_prefix[ns] = (uint32_t)tiles;
        samp_prefix[ns] = (uint32_t)sblocks;
        if (total_out > out_capacity) return GRAVAC_ERR_CAPACITY;
        if (tiles > max_tiles(n, ns) || sblocks > max_sample_blocks(n, ns)) return GRAVAC_ERR_WORKSPACE;
        p.n_tiles = (uint32_t)tiles;
        p.n_sample_blocks = (uint32_t)sblocks;
        hipError_t e = hipSuccess;
        auto up = [&](size_t off, const void* src, size_t bytes) {
            if (e == hipSuccess) e = hipMemcpyAsync(ws + off, src, bytes, hipMemcpyHostToDevice, stream);
        };
        up(L.seg_off, seg_offsets, sizeof(int64_t) * (ns + 1));
        up(L.koff, koff.data(), sizeof(int64_t) * (ns + 1));
        up(L.tile_prefix, tile_prefix.data(), sizeof(uint32_t) * (ns + 1));
        up(L.samp_prefix, samp_prefix.data(), sizeof(uint32_t) * (ns + 1));
        up(L.samp_cnt, samp_cnt.data(), sizeof(uint32_t) * ns);
        up(L.ktab, ktab.data(), sizeof(uint32_t) * (size_t)ns * n_cf);
        if (e != hipSuccess) return GRAVAC_ERR_HIP;
        // the host vectors die at the end of this scope: wait for the copies (pageable memory is
        // staged by the runtime, but the guarantee is only given by a synchronisation)
        if (hipStreamSynchronize(stream) != hipSuccess) return GRAVAC_ERR_HIP;
    }

    const int cus = device_cus();
    const uint32_t tile_wgs = (p.n_tiles + WAVES - 1) / WAVES;
    const uint32_t stream_grid = tile_wgs < (uint32_t)cus * 8 ? tile_wgs : (uint32_t)cus * 8;
    const uint32_t light_grid = tile_wgs < (uint32_t)cus * 4 ? tile_wgs : (uint32_t)cus * 4;
    const dim3 per_cf(ns, n_cf);

    const bool prof = (flags & GRAVAC_FLAG_PROFILE) != 0;
    if (prof) {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        if (!g_ev_ready) {
            for (int i = 0; i < 4; ++i)
                if (hipEventCreate(&g_ev[i]) != hipSuccess) return GRAVAC_ERR_HIP;
            g_ev_ready = true;
        }
        (void)hipEventRecord(g_ev[0], stream);
    }
    hipLaunchKernelGGL(sample_kernel, dim3(p.n_sample_blocks), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(threshold_kernel, dim3(ns), dim3(1024), 0, stream, p);
    if (prof) (void)hipEventRecord(g_ev[1], stream);
    hipLaunchKernelGGL(stream_kernel<true>, dim3(stream_grid), dim3(WG), 0, stream, p);
    if (prof) (void)hipEventRecord(g_ev[2], stream);
    hipLaunchKernelGGL(locate_kernel, per_cf, dim3(256), 0, stream, p, 0);
    // exact route, taken only by segments whose sampled bound failed
    hipLaunchKernelGGL(coarse_kernel, dim3(stream_grid), dim3(WG), 0, stream, p);
    hipLaunchKernelGGL(locate_coarse_kernel, per_cf, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(stream_kernel<false>, dim3(stream_grid), dim3(WG), 0, stream, p);
    hipLaunchKernelGGL(locate_kernel, per_cf, dim3(256), 0, stream, p, 1);
    // exact resolution on the candidates
    hipLaunchKernelGGL(refine_kernel, dim3(light_grid), dim3(WG), 0, stream, p);
    hipLaunchKernelGGL(resolve_kernel, per_cf, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(tile_count_kernel, dim3(light_grid), dim3(WG), 0, stream, p);
    hipLaunchKernelGGL(scan_kernel, dim3(ns, 1 + n_cf), dim3(ns == 1 ? 1024 : 256), 0, stream, p);
    hipLaunchKernelGGL(emit_kernel, dim3(light_grid), dim3(WG), 0, stream, p);
    if (prof) {
        (void)hipEventRecord(g_ev[3], stream);
        g_ev_recorded = true;
    }
    if (hipGetLastError() != hipSuccess) return GRAVAC_ERR_HIP;
    return GRAVAC_OK;
}

int gravac_decompress_accumulate(const int32_t* idx, const float* val, const int64_t* counts, int W, int64_t n,
                                 float* dense_out, void* stream_v)
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
    const int cus = device_cus();
    const int64_t ntile = (n + DTILE - 1) / DTILE;
    const uint32_t grid = (uint32_t)(ntile < (int64_t)cus * 16 ? ntile : (int64_t)cus * 16);
    int64_t at = 0;
    for (int w0 = 0; w0 < W; w0 += DMAXW) {
        const int wn = (W - w0 < DMAXW) ? W - w0 : DMAXW;
        WorkerOffsets wo;
        int64_t group = 0;
        for (int w = 0; w < wn; ++w) {
            wo.at[w] = at + group;
            group += counts[w0 + w];
        }
        for (int w = wn; w <= DMAXW; ++w) wo.at[w] = at + group;
        at += group;
        if (group == 0) continue;
        hipLaunchKernelGGL(decompress_kernel, dim3(grid), dim3(256), 0, stream, idx, val, wo, wn, n, dense_out);
    }
    if (hipGetLastError() != hipSuccess) return GRAVAC_ERR_HIP;
    return GRAVAC_OK;
}

int gravac_read_status(const void* workspace, void* stream_v, int32_t* out8)
{
    if (!workspace || !out8) return GRAVAC_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_v;
    if (hipStreamSynchronize(stream) != hipSuccess) return GRAVAC_ERR_HIP;
    Status s;
    if (hipMemcpy(&s, workspace, sizeof(Status), hipMemcpyDeviceToHost) != hipSuccess) return GRAVAC_ERR_HIP;
    out8[0] = s.any_fail; out8[1] = s.n_fail; out8[2] = s.error; out8[3] = s.n_seg;
    out8[4] = out8[5] = out8[6] = out8[7] = 0;
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
        default: return "unknown error code";
    }
}

}  // extern "C"
