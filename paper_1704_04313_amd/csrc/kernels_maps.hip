// Memory-bound kernels of the change-based convolution layer for gfx950 (wave64):
// change detection, dilation by the filter support, change-index extraction, sparse
// max-pooling and the final layout change.  See kernels.h for the data layout.
#include "kernels.h"

namespace cbk {

static constexpr int kBlock = 256;

// ------------------------------------------------------------------------------------------
// Change detection on a planar frame.  A wave takes kDetectPix * 64 consecutive pixels, lane l
// the pixels l, l + 64, ...: every access is a full-wave coalesced transaction (one channel
// plane of the frame, or one 16-byte unit per lane of the stored map), and the loads of all
// of a lane's pixels are issued before the first is used, which is what keeps enough bytes in
// flight to approach the HBM rate.  Each group of 64 pixels yields one word of the change bitmap.
// ------------------------------------------------------------------------------------------
static constexpr int kDetectPix = 4;

template <int DT, int HOLD>
__global__ __launch_bounds__(kBlock) void detect_frame_kernel(const float *__restrict__ frame,
                                                              uint4 *__restrict__ ref, uint4 *__restrict__ cur,
                                                              uint64_t *__restrict__ bits, int C, int V, int N,
                                                              int total, float tau, int force,
                                                              uint64_t *__restrict__ clear, long long clear_words)
{
    constexpr int E = Unit<DT>::N;
    constexpr int P = kDetectPix;
    const int tid = blockIdx.x * kBlock + threadIdx.x;
    for (long long i = tid; i < clear_words; i += (long long)gridDim.x * kBlock) clear[i] = 0ull;
    const int lane = threadIdx.x & 63;
    const int g0 = (tid >> 6) * (64 * P) + lane; // this lane's first pixel
    bool ok[P], flag[P];
    const float *fp[P];
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int g = g0 + 64 * k;
        ok[k] = g < total;
        flag[k] = false;
        const int st = ok[k] ? g / N : 0;
        fp[k] = frame + (size_t)st * C * N + (ok[k] ? g - st * N : 0);
    }
    for (int u = 0; u < V; ++u) {
        uint4 xv[P], rv[P];
#pragma unroll
        for (int k = 0; k < P; ++k) {
            xv[k] = make_uint4(0u, 0u, 0u, 0u);
            rv[k] = xv[k];
            if (ok[k]) {
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    const int c = u * E + i;
                    if (c < C) Unit<DT>::set(xv[k], i, fp[k][(size_t)c * N]);
                }
                if (!force) rv[k] = ref[(size_t)(g0 + 64 * k) * V + u];
            }
        }
#pragma unroll
        for (int k = 0; k < P; ++k) {
            if (!ok[k]) continue;
            if (!force) flag[k] |= unit_exceeds<DT>(xv[k], rv[k], tau);
            if (HOLD)
                cur[(size_t)(g0 + 64 * k) * V + u] = xv[k];
            else
                ref[(size_t)(g0 + 64 * k) * V + u] = xv[k];
        }
    }
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int g = g0 + 64 * k;
        if (force) flag[k] = ok[k];
        if (HOLD && flag[k])
            for (int u = 0; u < V; ++u) ref[(size_t)g * V + u] = cur[(size_t)g * V + u];
        const uint64_t word = __ballot(flag[k]);
        if (lane == 0 && g < total) bits[g >> 6] = word;
    }
}

hipError_t detect_frame(hipStream_t st, const float *frame, void *ref, void *cur, uint64_t *bits, int C, int V,
                        int N, int S, float tau, int hold, int force, int dtype, uint64_t *clear,
                        long long clear_words, const Timing &tm)
{
    if (!clear) clear_words = 0;
    const int total = S * N;
    const int grid = (total + kBlock * kDetectPix - 1) / (kBlock * kDetectPix);
    uint4 *r = static_cast<uint4 *>(ref), *c = static_cast<uint4 *>(cur);
#define CBK_LAUNCH(DT_, HOLD_)                                                                                  \
    launch_kernel(tm, detect_frame_kernel<DT_, HOLD_>, dim3(grid), dim3(kBlock), 0, st, frame, r, c, bits, C, \
                       V, N, total, tau, force, clear, clear_words)
    if (dtype == kBF16) {
        if (hold) CBK_LAUNCH(kBF16, 1); else CBK_LAUNCH(kBF16, 0);
    } else {
        if (hold) CBK_LAUNCH(kF32, 1); else CBK_LAUNCH(kF32, 0);
    }
#undef CBK_LAUNCH
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Change detection map against map.  One workgroup per 64 pixels (one bitmap word); its
// waves take turns over the 64*V units of those pixels, so every access is a fully
// coalesced 1 KiB wave transaction.  A wave-wide ballot of "this unit exceeded" is folded
// into per-pixel flags by masking the ballot with each pixel's unit range.
// ------------------------------------------------------------------------------------------
template <int DT, int HOLD>
__global__ __launch_bounds__(1024) void detect_map_kernel(const uint4 *__restrict__ x, uint4 *__restrict__ ref,
                                                          uint64_t *__restrict__ bits, int V, int total,
                                                          float tau, int force)
{
    __shared__ uint64_t swords[16];
    const int word = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int px0 = word * 64;
    const int npx = min(64, total - px0);
    const size_t base = (size_t)px0 * V;
    const int nf = npx * V;
    const int lo0 = lane * V;
    bool mine = false;
    for (int t = wave; t * 64 < nf; t += nw) {
        const int f = t * 64 + lane;
        bool e = false;
        if (f < nf) {
            const uint4 a = x[base + f];
            if (!force) e = unit_exceeds<DT>(a, ref[base + f], tau);
            if (!HOLD) ref[base + f] = a;
        }
        const uint64_t B = __ballot(e);
        int lo = lo0 - t * 64, hi = lo + V;
        lo = max(lo, 0);
        hi = min(hi, 64);
        if (lo < hi) {
            const int len = hi - lo;
            const uint64_t mask = (len >= 64) ? ~0ull : (((1ull << len) - 1ull) << lo);
            mine |= (B & mask) != 0ull;
        }
    }
    if (force) mine = lane < npx;
    uint64_t w = __ballot(mine);
    if (nw > 1) {
        if (lane == 0) swords[wave] = w;
        __syncthreads();
        w = 0;
        for (int i = 0; i < nw; ++i) w |= swords[i];
    }
    if (threadIdx.x == 0) bits[word] = w;
    if (HOLD) {
        // refresh the stored input only at flagged pixels (all channels)
        for (int f = threadIdx.x; f < nf; f += blockDim.x) {
            const int px = f / V;
            if ((w >> px) & 1ull) ref[base + f] = x[base + f];
        }
    }
}

hipError_t detect_map(hipStream_t st, const void *x, void *ref, uint64_t *bits, int V, int total, float tau,
                      int hold, int force, int dtype, const Timing &tm)
{
    const int words = (total + 63) / 64;
    int nw = V < 16 ? V : 16;
    if (nw < 1) nw = 1;
    const uint4 *x4 = static_cast<const uint4 *>(x);
    uint4 *r4 = static_cast<uint4 *>(ref);
#define CBK_LAUNCH(DT_, HOLD_)                                                                                  \
    launch_kernel(tm, detect_map_kernel<DT_, HOLD_>, dim3(words), dim3(nw * 64), 0, st, x4, r4, bits, V, total, \
                       tau, force)
    if (dtype == kBF16) {
        if (hold) CBK_LAUNCH(kBF16, 1); else CBK_LAUNCH(kBF16, 0);
    } else {
        if (hold) CBK_LAUNCH(kF32, 1); else CBK_LAUNCH(kF32, 0);
    }
#undef CBK_LAUNCH
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Dilation.  An output position must be recomputed iff its receptive field contains a
// changed input position.  One thread per output position tests, for each of the kh rows
// of its field, the (clipped) run of kw bits of the change bitmap with two word reads.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t bit_run(const uint64_t *__restrict__ m, long long a, int len)
{
    const long long w = a >> 6;
    const int o = (int)(a & 63);
    uint64_t v = m[w] >> o;
    if (o + len > 64) v |= m[w + 1] << (64 - o);
    if (len < 64) v &= (1ull << len) - 1ull;
    return v;
}

// Same question for a map with one byte per pixel (nonzero = changed): is any of the len bytes
// starting at byte a set?  Eight bytes per step through two aligned 64-bit loads.
__device__ __forceinline__ bool byte_run_any(const uint64_t *__restrict__ m, long long a, int len)
{
    bool any = false;
    while (len > 0) {
        const int n = len < 8 ? len : 8;
        const long long w = a >> 3;
        const int o = (int)(a & 7) * 8;
        uint64_t v = m[w] >> o;
        if (o + n * 8 > 64) v |= m[w + 1] << (64 - o);
        if (n < 8) v &= (1ull << (n * 8)) - 1ull;
        any |= v != 0ull;
        a += n;
        len -= n;
    }
    return any;
}

template <bool BYTES>
__device__ __forceinline__ bool field_changed(const uint64_t *__restrict__ m, const DilateGeom &g, int st,
                                              int qy, int qx)
{
    const int x0 = max(qx * g.stride - g.pad, 0);
    const int x1 = min(qx * g.stride - g.pad + g.kw - 1, g.W - 1);
    if (x0 > x1) return false;
    const int len = x1 - x0 + 1;
    bool any = false;
    for (int j = 0; j < g.kh; ++j) {
        const int iy = qy * g.stride - g.pad + j;
        if ((unsigned)iy < (unsigned)g.H) {
            const long long a = ((long long)st * g.H + iy) * g.W + x0;
            if (BYTES)
                any |= byte_run_any(m, a, len);
            else
                any |= bit_run(m, a, len) != 0ull;
        }
    }
    return any;
}

template <bool BYTES>
__global__ __launch_bounds__(kBlock) void dilate_kernel(const uint64_t *__restrict__ chg,
                                                        uint64_t *__restrict__ upd,
                                                        uint64_t *__restrict__ pool, DilateGeom g,
                                                        int upd_blocks)
{
    if ((int)blockIdx.x < upd_blocks) {
        const int No = g.Ho * g.Wo;
        const int total = g.S * No;
        const int t = blockIdx.x * kBlock + threadIdx.x;
        bool f = false;
        if (t < total) {
            const int st = t / No, q = t - st * No;
            const int qy = q / g.Wo, qx = q - qy * g.Wo;
            f = field_changed<BYTES>(chg, g, st, qy, qx);
        }
        const uint64_t word = __ballot(f);
        const int t0 = t & ~63;
        if ((threadIdx.x & 63) == 0 && t0 < total) upd[t0 >> 6] = word;
    } else {
        const int Np = g.Hp * g.Wp;
        const int total = g.S * Np;
        const int t = (blockIdx.x - upd_blocks) * kBlock + threadIdx.x;
        bool f = false;
        if (t < total) {
            const int st = t / Np, q = t - st * Np;
            const int py = q / g.Wp, px = q - py * g.Wp;
            DilateGeom e = g;
            e.stride = g.stride * g.pool_k;
            e.kh = g.kh + (g.pool_k - 1) * g.stride;
            e.kw = g.kw + (g.pool_k - 1) * g.stride;
            if (g.stride <= g.kh && g.stride <= g.kw && (BYTES || e.kw <= 64)) {
                // the k x k outputs' receptive fields tile one larger window without gaps
                f = field_changed<BYTES>(chg, e, st, py, px);
            } else {
                for (int a = 0; a < g.pool_k; ++a)
                    for (int b = 0; b < g.pool_k; ++b)
                        f |= field_changed<BYTES>(chg, g, st, py * g.pool_k + a, px * g.pool_k + b);
            }
        }
        const uint64_t word = __ballot(f);
        const int t0 = t & ~63;
        if ((threadIdx.x & 63) == 0 && t0 < total) pool[t0 >> 6] = word;
    }
}

hipError_t dilate(hipStream_t st, const uint64_t *chg_bits, uint64_t *upd_bits, uint64_t *pool_bits,
                  const DilateGeom &g, const Timing &tm)
{
    const int ub = (g.S * g.Ho * g.Wo + kBlock - 1) / kBlock;
    const int pb = (pool_bits && g.pool_k > 0) ? (g.S * g.Hp * g.Wp + kBlock - 1) / kBlock : 0;
    if (g.chg_bytes)
        launch_kernel(tm, dilate_kernel<true>, dim3(ub + pb), dim3(kBlock), 0, st, chg_bits, upd_bits, pool_bits, g,
                           ub);
    else
        launch_kernel(tm, dilate_kernel<false>, dim3(ub + pb), dim3(kBlock), 0, st, chg_bits, upd_bits, pool_bits, g,
                           ub);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Change-index extraction.  Each workgroup owns kCompactWords bitmap words.  It obtains its
// output offset by counting the set bits of all preceding words itself (the bitmaps are a
// few KiB to a few hundred KiB and L2 resident, so this is cheaper and simpler than a second
// launch or a cross-workgroup handshake, and it is deterministic), scans its own words'
// popcounts, expands the bits into an LDS staging buffer and copies that out coalesced.
// ------------------------------------------------------------------------------------------
static constexpr int kCompactWords = 128;

struct CompactJobs {
    CompactJob j[3];
};

__device__ __forceinline__ int wave_incl_scan(int v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// Word i (64 pixels) of a job's map as a bit mask.  A byte map (one byte per pixel, nonzero =
// set) is packed on the fly: the high bit of (x | (x & 0x7f..7f) + 0x7f..7f) marks nonzero bytes,
// and the multiplication gathers those eight marks into one byte.
__device__ __forceinline__ uint64_t map_word(const CompactJob &job, int i)
{
    if (!job.bytes) return job.bits[i];
    uint64_t w = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint64_t x = job.bits[(size_t)i * 8 + k];
        const uint64_t nz = ((x | ((x & 0x7f7f7f7f7f7f7f7full) + 0x7f7f7f7f7f7f7f7full)) & 0x8080808080808080ull) >> 7;
        w |= ((nz * 0x0102040810204080ull) >> 56) << (8 * k);
    }
    return w;
}

// Set bits per workgroup-sized group of words, for maps with so many groups that letting every
// workgroup recount all preceding words would dominate (see compact_kernel).
__global__ __launch_bounds__(kBlock) void compact_count_kernel(CompactJobs jobs)
{
    __shared__ int swave[4];
    const CompactJob job = jobs.j[blockIdx.y];
    const int w0 = blockIdx.x * kCompactWords;
    if (w0 >= job.nwords) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int c = 0;
    if (tid < kCompactWords && w0 + tid < job.nwords) c = __popcll(map_word(job, w0 + tid));
    c = wave_incl_scan(c, lane);
    if (lane == 63) swave[wave] = c;
    __syncthreads();
    if (tid == 0) job.group_counts[blockIdx.x] = swave[0] + swave[1] + swave[2] + swave[3];
}

template <bool TWO_LEVEL>
__global__ __launch_bounds__(kBlock) void compact_kernel(CompactJobs jobs)
{
    __shared__ int stage[kCompactWords * 64];
    __shared__ int swave[4];
    __shared__ int swave2[4];
    const CompactJob job = jobs.j[blockIdx.y];
    const int w0 = blockIdx.x * kCompactWords;
    if (w0 >= job.nwords) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // set bits in all words before this workgroup's
    int before = 0;
    if (TWO_LEVEL) {
        for (int i = tid; i < (int)blockIdx.x; i += kBlock) before += job.group_counts[i];
    } else {
        for (int i = tid; i < w0; i += kBlock) before += __popcll(map_word(job, i));
    }
    before = wave_incl_scan(before, lane);
    if (lane == 63) swave[wave] = before;

    // this workgroup's words, one per thread of the first two waves
    uint64_t mine = 0;
    if (tid < kCompactWords && w0 + tid < job.nwords) mine = map_word(job, w0 + tid);
    const int cnt = __popcll(mine);
    const int incl = wave_incl_scan(cnt, lane);
    if (lane == 63) swave2[wave] = incl;
    __syncthreads();
    const int prefix = swave[0] + swave[1] + swave[2] + swave[3];
    int off = incl - cnt;
    for (int i = 0; i < wave; ++i) off += swave2[i];
    const int total = swave2[0] + swave2[1] + swave2[2] + swave2[3];

    const int pos0 = (w0 + tid) * 64;
    while (mine) {
        const int b = __ffsll((unsigned long long)mine) - 1;
        stage[off++] = pos0 + b;
        mine &= mine - 1ull;
    }
    __syncthreads();
    for (int i = tid; i < total; i += kBlock) job.list[prefix + i] = stage[i];
    if (tid == 0 && w0 + kCompactWords >= job.nwords) *job.count = prefix + total;
}

bool compact_two_level(int nwords) { return nwords > kCompactWords * 48; }

size_t compact_group_count_bytes(int nwords) { return ((size_t)nwords / kCompactWords + 2) * sizeof(int); }

hipError_t compact(hipStream_t st, const CompactJob *jobs, int njobs, const Timing &tm)
{
    if (njobs < 1 || njobs > 3) return hipErrorInvalidValue;
    CompactJobs js;
    int maxw = 1;
    for (int i = 0; i < 3; ++i) {
        js.j[i] = jobs[i < njobs ? i : 0];
        if (i < njobs && jobs[i].nwords > maxw) maxw = jobs[i].nwords;
    }
    const int gx = (maxw + kCompactWords - 1) / kCompactWords;
    if (compact_two_level(maxw)) {
        for (int i = 0; i < njobs; ++i)
            if (!jobs[i].group_counts) return hipErrorInvalidValue;
        launch_kernel(Timing{tm.start, nullptr}, compact_count_kernel, dim3(gx, njobs), dim3(kBlock), 0, st, js);
        launch_kernel(Timing{nullptr, tm.stop}, compact_kernel<true>, dim3(gx, njobs), dim3(kBlock), 0, st, js);
    } else {
        launch_kernel(tm, compact_kernel<false>, dim3(gx, njobs), dim3(kBlock), 0, st, js);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Max-pooling at the listed pooled positions only: each is the maximum over its k x k window
// of the stored (already updated, post-activation) map.  One thread per (position, 16-byte unit of channels).
// ------------------------------------------------------------------------------------------
// One pooled position g, one unit v of its channels: the maximum over the window, the optional
// comparison with the value it replaces (all lanes of the wave must call this together: the
// flag of a position is combined across its V lanes with a ballot when V is a power of two).
template <int DT>
__device__ __forceinline__ void pool_unit(bool active, int g, int v, const uint4 *__restrict__ in,
                                          uint4 *__restrict__ pooled, int V, int k, int Wo, int No, int Wp, int Np,
                                          unsigned char *__restrict__ next_flags, float next_tau, int next_force)
{
    const int lane = threadIdx.x & 63;
    const bool pow2 = (V & (V - 1)) == 0 && V <= 64;
    uint4 m = make_uint4(0u, 0u, 0u, 0u);
    bool f = false;
    if (active) {
        const int st = g / Np, pp = g - st * Np;
        const int py = pp / Wp, px = pp - py * Wp;
        const long long base = (long long)st * No + (long long)(py * k) * Wo + px * k;
        m = in[base * V + v];
        for (int j = 0; j < k; ++j)
            for (int i = 0; i < k; ++i) m = unit_max<DT>(m, in[(base + (long long)j * Wo + i) * V + v]);
        if (next_flags) {
            // Change detection of the layer this map feeds (Section 3.1, first formula): the value
            // being replaced is that layer's stored previous input, and positions that are not
            // recomputed cannot differ from it.
            f = next_force != 0;
            if (!f) f = unit_exceeds<DT>(m, pooled[(long long)g * V + v], next_tau);
        }
    }
    if (next_flags) {
        if (pow2) {
            const unsigned long long B = __ballot(f);
            const unsigned long long grp = (V == 64) ? ~0ull : (((1ull << V) - 1ull) << (lane & ~(V - 1)));
            if (active && v == 0 && (B & grp) != 0ull) next_flags[g] = 1;
        } else if (f) {
            next_flags[g] = 1;
        }
    }
    if (active) pooled[(long long)g * V + v] = m;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void pool_sparse_kernel(const int *__restrict__ list,
                                                             const int *__restrict__ count,
                                                             const uint4 *__restrict__ in,
                                                             uint4 *__restrict__ pooled, int V, int k, int Wo,
                                                             int No, int Wp, int Np,
                                                             unsigned char *__restrict__ next_flags,
                                                             float next_tau, int next_force)
{
    const long long total = (long long)(*count) * V;
    const long long step = (long long)gridDim.x * kBlock;
    // whole waves iterate together (the last round with some lanes inactive)
    for (long long i0 = (long long)blockIdx.x * kBlock; i0 < total; i0 += step) {
        const long long idx = i0 + threadIdx.x;
        const bool active = idx < total;
        const int u = active ? (int)(idx / V) : 0, v = active ? (int)(idx - (long long)u * V) : 0;
        const int g = active ? list[u] : 0;
        pool_unit<DT>(active, g, v, in, pooled, V, k, Wo, No, Wp, Np, next_flags, next_tau, next_force);
    }
}

template <int DT>
__global__ __launch_bounds__(kBlock) void pool_masked_kernel(const uint64_t *__restrict__ bits, int from_outputs,
                                                             int total_px,
                                                             const uint4 *__restrict__ in,
                                                             uint4 *__restrict__ pooled, int V, int k, int Wo,
                                                             int No, int Wp, int Np,
                                                             unsigned char *__restrict__ next_flags,
                                                             float next_tau, int next_force)
{
    const long long total = (long long)total_px * V;
    const long long step = (long long)gridDim.x * kBlock;
    for (long long i0 = (long long)blockIdx.x * kBlock; i0 < total; i0 += step) {
        const long long idx = i0 + threadIdx.x;
        bool active = idx < total;
        const int g = active ? (int)(idx / V) : 0, v = active ? (int)(idx - (long long)g * V) : 0;
        if (active) {
            if (from_outputs) {
                const int st = g / Np, pp = g - st * Np;
                const int py = pp / Wp, px = pp - py * Wp;
                bool any = false;
                for (int j = 0; j < k; ++j) {
                    const long long q0 = (long long)st * No + (long long)(py * k + j) * Wo + px * k;
                    for (int i = 0; i < k; ++i) any |= ((bits[(q0 + i) >> 6] >> ((q0 + i) & 63)) & 1ull) != 0ull;
                }
                active = any;
            } else {
                active = ((bits[g >> 6] >> (g & 63)) & 1ull) != 0ull;
            }
        }
        pool_unit<DT>(active, g, v, in, pooled, V, k, Wo, No, Wp, Np, next_flags, next_tau, next_force);
    }
}

hipError_t pool_sparse(hipStream_t st, const int *list, const int *count, int max_count, const void *in,
                       void *pooled, int V, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force, int dtype, const Timing &tm)
{
    long long work = (long long)max_count * V;
    long long grid = (work + kBlock - 1) / kBlock;
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    const uint4 *i4 = static_cast<const uint4 *>(in);
    uint4 *p4 = static_cast<uint4 *>(pooled);
    if (dtype == kBF16)
        launch_kernel(tm, pool_sparse_kernel<kBF16>, dim3((int)grid), dim3(kBlock), 0, st, list, count, i4, p4, V, k,
                           Wo, No, Wp, Np, next_flags, next_tau, next_force);
    else
        launch_kernel(tm, pool_sparse_kernel<kF32>, dim3((int)grid), dim3(kBlock), 0, st, list, count, i4, p4, V, k,
                           Wo, No, Wp, Np, next_flags, next_tau, next_force);
    return hipGetLastError();
}

hipError_t pool_masked(hipStream_t st, const uint64_t *bits, int from_outputs, int total, const void *in,
                       void *pooled, int V, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force, int dtype, const Timing &tm)
{
    long long work = (long long)total * V;
    long long grid = (work + kBlock - 1) / kBlock;
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    const uint4 *i4 = static_cast<const uint4 *>(in);
    uint4 *p4 = static_cast<uint4 *>(pooled);
    if (dtype == kBF16)
        launch_kernel(tm, pool_masked_kernel<kBF16>, dim3((int)grid), dim3(kBlock), 0, st, bits, from_outputs, total, i4, p4, V, k,
                           Wo, No, Wp, Np, next_flags, next_tau, next_force);
    else
        launch_kernel(tm, pool_masked_kernel<kF32>, dim3((int)grid), dim3(kBlock), 0, st, bits, from_outputs, total, i4, p4, V, k,
                           Wo, No, Wp, Np, next_flags, next_tau, next_force);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Stored map [S*No][V units] -> planar float32 [S][M][No].  Consecutive lanes take consecutive
// pixels' units (16-byte reads) and write one contiguous run per channel plane.
// ------------------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kBlock) void map_to_planar_kernel(const uint4 *__restrict__ map,
                                                               float *__restrict__ planar, int M, int V,
                                                               int No, long long total)
{
    constexpr int E = Unit<DT>::N;
    for (long long idx = (long long)blockIdx.x * kBlock + threadIdx.x; idx < total;
         idx += (long long)gridDim.x * kBlock) {
        const int q = (int)(idx % No);
        const long long sv = idx / No;
        const int v = (int)(sv % V);
        const long long st = sv / V;
        const uint4 a = map[(st * No + q) * V + v];
        float *dst = planar + (st * M + (long long)E * v) * No + q;
#pragma unroll
        for (int i = 0; i < E; ++i)
            if (E * v + i < M) dst[(long long)i * No] = Unit<DT>::get(a, i);
    }
}

hipError_t map_to_planar(hipStream_t st, const void *map, float *planar, int M, int V, int No, int S, int dtype,
                         const Timing &tm)
{
    const long long total = (long long)S * V * No;
    long long grid = (total + kBlock - 1) / kBlock;
    if (grid > 8192) grid = 8192;
    if (grid < 1) grid = 1;
    const uint4 *m4 = static_cast<const uint4 *>(map);
    if (dtype == kBF16)
        launch_kernel(tm, map_to_planar_kernel<kBF16>, dim3((int)grid), dim3(kBlock), 0, st, m4, planar, M, V, No,
                           total);
    else
        launch_kernel(tm, map_to_planar_kernel<kF32>, dim3((int)grid), dim3(kBlock), 0, st, m4, planar, M, V, No,
                           total);
    return hipGetLastError();
}

__global__ void iota_kernel(int *list, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) list[i] = i;
}

hipError_t fill_iota(hipStream_t st, int *list, int n)
{
    int grid = (n + 255) / 256;
    if (grid > 1024) grid = 1024;
    if (grid < 1) grid = 1;
    launch_kernel(Timing(), iota_kernel, dim3(grid), dim3(256), 0, st, list, n);
    return hipGetLastError();
}

} // namespace cbk
