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
                                                              uint64_t *__restrict__ clear, long long clear_words,
                                                              FastDiv dN)
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
        const int st = ok[k] ? fast_div(g, dN) : 0;
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

// ------------------------------------------------------------------------------------------
// The same for a float32 map without padding channels (C = 1, 2, 3, 5, 6 or 7 values per pixel):
// the stored input then moves exactly the bytes the method needs (with three channels 12
// instead of 16 per pixel and direction).  A wave takes 256 consecutive pixels = 64 * C float4
// of the map.  Lane l reads its pixels l, l + 64, ... from the frame's planes as before and
// puts them into LDS in map order; from there every lane takes the float4 l, l + 64, ... of the
// wave's piece, compares them with the stored ones, marks the pixels of the elements that differ
// in an LDS flag array, and after that each lane collects the flags of its own pixels for the
// bitmap words.  All global accesses stay full-wave coalesced.
// ------------------------------------------------------------------------------------------
static constexpr int kPackMaxC = 7;

template <int HOLD>
__global__ __launch_bounds__(kBlock) void detect_frame_packed_kernel(const float *__restrict__ frame,
                                                                     float *__restrict__ ref, float *__restrict__ cur,
                                                                     uint64_t *__restrict__ bits, int C, int N,
                                                                     int total, float tau, int force,
                                                                     uint64_t *__restrict__ clear, long long clear_words,
                                                                     FastDiv dN)
{
    constexpr int P = kDetectPix;       // pixels per lane
    constexpr int WP = 64 * P;          // pixels per wave
    constexpr int WAVES = kBlock / 64;
    __shared__ __align__(16) float sX[WAVES][WP * kPackMaxC];
    __shared__ int sF[WAVES][WP];
    const int tid = blockIdx.x * kBlock + threadIdx.x;
    for (long long i = tid; i < clear_words; i += (long long)gridDim.x * kBlock) clear[i] = 0ull;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p0 = (tid >> 6) * WP; // the wave's first pixel
    float *sx = sX[wave];
    int *sf = sF[wave];
    const long long e0 = (long long)p0 * C;          // the wave's first map element (a multiple of 4)
    const long long e_end = (long long)total * C;    // elements of the whole map
    const int inv = (65536 + C - 1) / C;             // e / C == (e * inv) >> 16 for e < 256 * 7, C <= 7
    // all global loads first: the frame's values of this lane's pixels and its float4 of the stored map
    float fv[P][kPackMaxC];
    float4 xv[kPackMaxC], rv[kPackMaxC];
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int g = p0 + lane + 64 * k;
        const int st = g < total ? fast_div(g, dN) : 0;
        const float *fp = frame + (size_t)st * C * N + (g < total ? g - st * N : 0);
#pragma unroll
        for (int c = 0; c < kPackMaxC; ++c) fv[k][c] = (c < C && g < total) ? fp[(size_t)c * N] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < kPackMaxC; ++j) {
        rv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j >= C || force) continue;
        const long long e = e0 + 4ll * (lane + 64 * j);
        if (e + 4 <= e_end) {
            rv[j] = *reinterpret_cast<const float4 *>(ref + e);
        } else {
            if (e + 0 < e_end) rv[j].x = ref[e + 0];
            if (e + 1 < e_end) rv[j].y = ref[e + 1];
            if (e + 2 < e_end) rv[j].z = ref[e + 2];
        }
    }
    // frame values -> LDS in map order (pixel-major, C values each), back as float4 of the map
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int pl = lane + 64 * k;
        sf[pl] = (force && p0 + pl < total) ? 1 : 0;
#pragma unroll
        for (int c = 0; c < kPackMaxC; ++c)
            if (c < C) sx[pl * C + c] = fv[k][c];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kPackMaxC; ++j)
        xv[j] = j < C ? *reinterpret_cast<const float4 *>(sx + 4 * (lane + 64 * j)) : make_float4(0.f, 0.f, 0.f, 0.f);
    if (!force) {
#pragma unroll
        for (int j = 0; j < kPackMaxC; ++j) {
            if (j >= C) break;
            const int el = 4 * (lane + 64 * j); // element inside the wave's piece
            const long long e = e0 + el;
            if (e + 0 < e_end && fabsf(xv[j].x - rv[j].x) > tau) sf[((el + 0) * inv) >> 16] = 1;
            if (e + 1 < e_end && fabsf(xv[j].y - rv[j].y) > tau) sf[((el + 1) * inv) >> 16] = 1;
            if (e + 2 < e_end && fabsf(xv[j].z - rv[j].z) > tau) sf[((el + 2) * inv) >> 16] = 1;
            if (e + 3 < e_end && fabsf(xv[j].w - rv[j].w) > tau) sf[((el + 3) * inv) >> 16] = 1;
        }
    }
    __syncthreads();
    // the stored map: everything (hold: the current frame everywhere, the reference where flagged)
#pragma unroll
    for (int j = 0; j < kPackMaxC; ++j) {
        if (j >= C) break;
        const int el = 4 * (lane + 64 * j);
        const long long e = e0 + el;
        if (e >= e_end) continue;
        float4 nr = xv[j];
        if (HOLD) {
            if (!sf[((el + 0) * inv) >> 16]) nr.x = rv[j].x;
            if (!sf[((el + 1) * inv) >> 16]) nr.y = rv[j].y;
            if (!sf[((el + 2) * inv) >> 16]) nr.z = rv[j].z;
            if (!sf[((el + 3) * inv) >> 16]) nr.w = rv[j].w;
        }
        if (e + 4 <= e_end) {
            if (HOLD) *reinterpret_cast<float4 *>(cur + e) = xv[j];
            *reinterpret_cast<float4 *>(ref + e) = nr;
        } else { // the map's last elements: nothing may be written behind them
            const float xs[3] = {xv[j].x, xv[j].y, xv[j].z}, ns[3] = {nr.x, nr.y, nr.z};
            for (int i = 0; i < 3; ++i)
                if (e + i < e_end) {
                    if (HOLD) cur[e + i] = xs[i];
                    ref[e + i] = ns[i];
                }
        }
    }
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int pl = lane + 64 * k, g = p0 + pl;
        const uint64_t word = __ballot(sf[pl] != 0);
        if (lane == 0 && g < total) bits[g >> 6] = word;
    }
}

// Frames of fewer pixels stay with whole units: their pass is bound by latency, not by bytes, and
// the way through LDS costs more than the padding.
static constexpr long long kPackMinPixels = 1 << 18;

bool detect_frame_packs(int dtype, int C, long long pixels)
{
    return dtype == kF32 && C % 4 != 0 && C <= kPackMaxC && pixels >= kPackMinPixels;
}

hipError_t detect_frame(hipStream_t st, const float *frame, void *ref, void *cur, uint64_t *bits, int C, int V,
                        int N, int S, float tau, int hold, int force, int dtype, int packed, uint64_t *clear,
                        long long clear_words, const Timing &tm)
{
    if (!clear) clear_words = 0;
    const int total = S * N;
    const FastDiv dN = make_fastdiv(N > 0 ? N : 1);
    const int grid = (total + kBlock * kDetectPix - 1) / (kBlock * kDetectPix);
    if (packed) {
        if (!detect_frame_packs(dtype, C, total)) return hipErrorInvalidValue;
        float *r = static_cast<float *>(ref), *c = static_cast<float *>(cur);
        if (hold)
            launch_kernel(tm, detect_frame_packed_kernel<1>, dim3(grid), dim3(kBlock), 0, st, frame, r, c, bits, C, N, total,
                          tau, force, clear, clear_words, dN);
        else
            launch_kernel(tm, detect_frame_packed_kernel<0>, dim3(grid), dim3(kBlock), 0, st, frame, r, c, bits, C, N, total,
                          tau, force, clear, clear_words, dN);
        return hipGetLastError();
    }
    uint4 *r = static_cast<uint4 *>(ref), *c = static_cast<uint4 *>(cur);
#define CBK_LAUNCH(DT_, HOLD_)                                                                                  \
    launch_kernel(tm, detect_frame_kernel<DT_, HOLD_>, dim3(grid), dim3(kBlock), 0, st, frame, r, c, bits, C, \
                       V, N, total, tau, force, clear, clear_words, dN)
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

// ------------------------------------------------------------------------------------------
// Dilation a word at a time, for layers of stride 1 with filters up to 16 wide (and a 2 x 2
// pooling behind them, if any) and of stride 2 without pooling behind them (Section 3: a strided
// convolution drops the unused columns of the image matrix; here it keeps every other bit of the
// dilated row).  A workgroup produces kCountWords words of the update map or of
// the pooled map, or counts as many of the change map.  It first brings the input rows its
// outputs read -- a contiguous piece of the change map -- into LDS as bits (a byte map is packed
// on the way): one round of coalesced loads, everything after that reads LDS.  Eight lanes then
// share one 64-position word: lane r takes the input rows r, r + 8, ... of the receptive fields.
// Dilation is separable and OR commutes, so each lane ORs the raw change bits of its rows (a
// window of the outputs' columns plus the filter's reach), then the shifted copies of that
// window by doubling, and the eight partial words are OR-ed across the lanes.  The fields of the
// 2 x 2 outputs under a pooled position tile one (kh+1) x (kw+1) window, so the pooled map is a
// dilation with that window at stride 2.  The workgroup also leaves the number of set bits of
// its words, which is what the index extraction needs to place its output.
// ------------------------------------------------------------------------------------------
static constexpr int kCompactTwoLevelBytesFrom = 768; // byte maps of more words than this: set bits counted per group first
static constexpr int kCompactTwoWordsFrom = 65536; // maps of more words than this: two words per thread in the index extraction
static constexpr int kCompactStage = 2048; // list entries a workgroup stages in LDS (8 KiB); more go straight to the list
static constexpr int kCompactDense = 12;   // words with more set bits than this are expanded by a whole wave
static constexpr int kCountWords = 32;    // words per entry of the group-count arrays
static constexpr int kWordLanes = 8;
static constexpr int kRegionWords = 4096; // LDS bitmap of the input piece: 32 KiB
static_assert(kCountWords * kWordLanes == kBlock, "one word per eight lanes");

// Bits [a, a + len) of the LDS bitmap as the low bits of the result; 1 <= len <= 64; the word
// behind the one holding bit a is read too (zero words follow the piece).
__device__ __forceinline__ uint64_t lds_run(const uint64_t *m, int a, int len)
{
    const int w = a >> 6, o = a & 63;
    const uint64_t lo = m[w], hi = m[w + 1];
    const uint64_t v = (lo >> o) | ((hi << 1) << (63 - o));
    return v & (~0ull >> (64 - len));
}

// A window of up to 192 columns, bit t = column xs + t.
struct Window {
    uint64_t w[3];
};

// OR over the input rows iy0 + j0, iy0 + j0 + dj, ... (j < nrows, inside the image) of stream st,
// columns xs .. xs + L - 1 (zero outside the image); L <= 192.  sM holds the change bits from
// position bit0 on.
__device__ __forceinline__ Window rows_or(const uint64_t *sM, int bit0, const DilateGeom &g, int st, int iy0,
                                          int nrows, int xs, int L, int j0, int dj)
{
    Window r = {{0ull, 0ull, 0ull}};
    const int k0 = xs < 0 ? -xs : 0, k1 = L < g.W - xs ? L : g.W - xs; // window bits inside the image
    for (int j = j0; j < nrows; j += dj) {
        const int iy = iy0 + j;
        if ((unsigned)iy >= (unsigned)g.H) continue;
        const int base = (st * g.H + iy) * g.W + xs - bit0;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const int lo = k0 > 64 * c ? k0 : 64 * c, hi = k1 < 64 * c + 64 ? k1 : 64 * c + 64;
            if (hi > lo) r.w[c] |= lds_run(sM, base + lo, hi - lo) << (lo - 64 * c);
        }
    }
    return r;
}

// bit t := OR of bits t .. t + taps - 1, by doubling
__device__ __forceinline__ void spread(Window &r, int taps)
{
    auto step = [&](int s) {
        r.w[0] |= (r.w[0] >> s) | (r.w[1] << (64 - s));
        r.w[1] |= (r.w[1] >> s) | (r.w[2] << (64 - s));
        r.w[2] |= r.w[2] >> s;
    };
    int cover = 1;
    while (cover * 2 <= taps) {
        step(cover);
        cover *= 2;
    }
    if (cover < taps) step(taps - cover);
}

// bits 0, 2, 4, ... of x moved to bits 0, 1, 2, ...
__device__ __forceinline__ uint64_t even_bits(uint64_t x)
{
    x &= 0x5555555555555555ull;
    x = (x | (x >> 1)) & 0x3333333333333333ull;
    x = (x | (x >> 2)) & 0x0f0f0f0f0f0f0f0full;
    x = (x | (x >> 4)) & 0x00ff00ff00ff00ffull;
    x = (x | (x >> 8)) & 0x0000ffff0000ffffull;
    x = (x | (x >> 16)) & 0x00000000ffffffffull;
    return x;
}

// OR over the kWordLanes lanes that share a word
__device__ __forceinline__ uint64_t word_lanes_or(uint64_t v)
{
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
#pragma unroll
    for (int d = 1; d < kWordLanes; d <<= 1) {
        lo |= (unsigned)__shfl_xor((int)lo, d, 64);
        hi |= (unsigned)__shfl_xor((int)hi, d, 64);
    }
    return ((uint64_t)hi << 32) | lo;
}

// eight bytes of a byte map -> eight bits: the high bit of (x | (x & 0x7f..7f) + 0x7f..7f) marks
// a nonzero byte and the multiplication gathers the eight marks
__device__ __forceinline__ unsigned nonzero_bytes(uint64_t x)
{
    const uint64_t nz = ((x | ((x & 0x7f7f7f7f7f7f7f7full) + 0x7f7f7f7f7f7f7f7full)) & 0x8080808080808080ull) >> 7;
    return (unsigned)((nz * 0x0102040810204080ull) >> 56);
}

struct DilateWords {
    const uint64_t *chg;
    uint64_t *upd, *pool;
    int *upd_groups, *pool_groups, *chg_groups; // all null: no counting
    DilateGeom g;
    FastDiv dWo, dHo, dWp, dHp;
    int upd_words, pool_words, chg_words;
    int upd_blocks, pool_blocks; // workgroups per role, in this order; the rest count the change map
    int region_words;            // capacity of the LDS piece in words
};

template <bool BYTES>
__global__ __launch_bounds__(kBlock) void dilate_words_kernel(DilateWords a)
{
    extern __shared__ uint64_t sM[]; // region_words + 2 words: the piece of the change map this workgroup reads
    __shared__ int swave[kBlock / 64];
    const DilateGeom &g = a.g;
    const int tid = threadIdx.x, r = tid & (kWordLanes - 1);
    int b = blockIdx.x;
    const int role = b < a.upd_blocks ? 0 : (b < a.upd_blocks + a.pool_blocks ? 1 : 2);
    if (role >= 1) b -= a.upd_blocks;
    if (role == 2) b -= a.pool_blocks;
    const int nwords = role == 0 ? a.upd_words : (role == 1 ? a.pool_words : a.chg_words);
    int *groups = role == 0 ? a.upd_groups : (role == 1 ? a.pool_groups : a.chg_groups);
    const int i = b * kCountWords + (tid >> 3); // this lane's word (shared with seven neighbours)
    uint64_t word = 0;

    if (role < 2) {
        // ---- the piece of the change map these words read, as bits in LDS
        const int per = role == 0 ? g.Wo : g.Wp, rows = role == 0 ? g.Ho : g.Hp;
        const FastDiv &dper = role == 0 ? a.dWo : a.dWp, &drows = role == 0 ? a.dHo : a.dHp;
        const int total = g.S * rows * per;
        const int q_lo = b * kCountWords * 64;
        const int q_hi = (q_lo + kCountWords * 64 < total ? q_lo + kCountWords * 64 : total) - 1;
        // first and last row (stream * rows + y) of those positions, then their first and last input row
        const int r_lo = fast_div(q_lo, dper), r_hi = fast_div(q_hi, dper);
        const int st_lo = fast_div(r_lo, drows), st_hi = fast_div(r_hi, drows);
        const int y_lo = r_lo - st_lo * rows, y_hi = r_hi - st_hi * rows;
        // a row (column) of this map steps `up` input rows (columns) and reads nrows (ncols) of them:
        // the filter's own reach for the update map of a layer of stride 1 or 2; for the pooled map
        // (stride-1 layers only) the kh + 1 rows that the 2 x 2 outputs under a pooled position tile
        const int up = role == 0 ? g.stride : 2;
        const int nrows = role == 0 ? g.kh : g.kh + 1;
        const int iy_lo = up * y_lo - g.pad > 0 ? up * y_lo - g.pad : 0;
        int iy_hi = up * y_hi - g.pad + nrows - 1;
        if (iy_hi > g.H - 1) iy_hi = g.H - 1;
        const int w_lo = ((st_lo * g.H + iy_lo) * g.W) >> 6;
        int w_hi = (((st_hi * g.H + iy_hi) * g.W + g.W - 1) >> 6) + 1; // one past the last word
        if (w_hi > a.chg_words) w_hi = a.chg_words;
        int nw = w_hi - w_lo;
        if (nw > a.region_words) nw = a.region_words; // the host sizes the LDS for the largest piece
        const int bit0 = w_lo * 64;
        if (BYTES) {
            unsigned char *sB = reinterpret_cast<unsigned char *>(sM);
            for (int k = tid; k < nw * 8; k += kBlock) sB[k] = (unsigned char)nonzero_bytes(a.chg[(size_t)w_lo * 8 + k]);
        } else {
            for (int k = tid; k < nw; k += kBlock) sM[k] = a.chg[w_lo + k];
        }
        if (tid < 2) sM[nw + tid] = 0ull;
        __syncthreads();

        if (i < nwords) { // the same for the lanes that share the word
            const int p0 = i * 64, p1 = p0 + 64 < total ? p0 + 64 : total;
            int pos = p0;
            const int row = fast_div(pos, dper);
            int x = pos - row * per, st = fast_div(row, drows), y = row - st * rows;
            while (pos < p1) { // one piece of a row at a time
                const int len = per - x < p1 - pos ? per - x : p1 - pos;
                uint64_t bits;
                if (role == 0 && g.stride == 1) {
                    Window wd = rows_or(sM, bit0, g, st, y - g.pad, g.kh, x - g.pad, len + g.kw - 1, r, kWordLanes);
                    spread(wd, g.kw);
                    bits = wd.w[0];
                } else if (role == 0) { // stride 2: the dilation at every input column, then every other bit
                    Window wd = rows_or(sM, bit0, g, st, 2 * y - g.pad, g.kh, 2 * x - g.pad, 2 * (len - 1) + g.kw, r,
                                        kWordLanes);
                    spread(wd, g.kw);
                    bits = even_bits(wd.w[0]) | (even_bits(wd.w[1]) << 32);
                } else {
                    Window wd = rows_or(sM, bit0, g, st, 2 * y - g.pad, g.kh + 1, 2 * x - g.pad, 2 * len + g.kw - 1, r,
                                        kWordLanes);
                    spread(wd, g.kw + 1);
                    bits = even_bits(wd.w[0]) | (even_bits(wd.w[1]) << 32);
                }
                if (len < 64) bits &= (1ull << len) - 1ull;
                word |= bits << (pos - p0);
                pos += len;
                x = 0;
                if (++y == rows) {
                    y = 0;
                    ++st;
                }
            }
        }
    } else if (i < nwords) {
        if (BYTES) // lane r packs positions 8r .. 8r+7 (the byte maps are padded to whole words)
            word = (uint64_t)nonzero_bytes(a.chg[(size_t)i * 8 + r]) << (8 * r);
        else if (r == 0)
            word = a.chg[i];
    }
    word = word_lanes_or(word);
    int count = 0;
    if (r == 0 && i < nwords) {
        if (role == 0) a.upd[i] = word;
        if (role == 1) a.pool[i] = word;
        count = __popcll(word);
    }
    if (!groups) return;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) count += __shfl_xor(count, d, 64);
    if ((tid & 63) == 0) swave[tid >> 6] = count;
    __syncthreads();
    if (tid == 0 && b * kCountWords < nwords) {
        int c = 0;
        for (int w = 0; w < kBlock / 64; ++w) c += swave[w];
        groups[b] = c;
    }
}

// Words of the change map that kCountWords output words (pooled: every pooled position stands
// for two rows and columns of outputs) can need at most.
static long long dilate_region_words(const DilateGeom &g, bool pooled)
{
    const long long per = pooled ? g.Wp : g.Wo, rows_per_stream = pooled ? g.Hp : g.Ho;
    const long long out_rows = (long long)kCountWords * 64 / per + 2; // rows touched by that many positions
    const long long streams = out_rows / rows_per_stream + 2;         // streams those rows can span
    // outputs' own rows, the filter's reach at both ends, and per stream boundary crossed the
    // rows by which a stream's input is taller than the output rows that count here; never more
    // than all input rows of those streams
    long long in_rows = (pooled ? 2 : g.stride) * out_rows + (g.kh + 2) * (streams + 1);
    if (in_rows > (streams + 1) * g.H) in_rows = (streams + 1) * g.H;
    return in_rows * g.W / 64 + 2;
}

bool dilate_counts(const DilateGeom &g)
{
    return (g.stride == 1 || (g.stride == 2 && g.pool_k == 0)) && g.kw >= 1 && g.kw <= 16 && g.kh >= 1 &&
           (g.pool_k == 0 || g.pool_k == 2) &&
           (long long)g.S * g.H * g.W < (1ll << 31) && (long long)g.S * g.Ho * g.Wo < (1ll << 31) &&
           dilate_region_words(g, false) <= kRegionWords && (g.pool_k == 0 || dilate_region_words(g, true) <= kRegionWords);
}

hipError_t dilate(hipStream_t st, const uint64_t *chg_bits, uint64_t *upd_bits, uint64_t *pool_bits,
                  const DilateGeom &g, const DilateGroups *groups, const Timing &tm)
{
    const bool pooled = pool_bits && g.pool_k > 0;
    if (dilate_counts(g)) {
        const bool count = groups && groups->upd && groups->chg && (!pooled || groups->pool);
        DilateWords a;
        a.chg = chg_bits; a.upd = upd_bits; a.pool = pooled ? pool_bits : nullptr;
        a.upd_groups = count ? groups->upd : nullptr;
        a.pool_groups = count ? groups->pool : nullptr;
        a.chg_groups = count ? groups->chg : nullptr;
        a.g = g;
        a.dWo = make_fastdiv(g.Wo); a.dHo = make_fastdiv(g.Ho);
        a.dWp = make_fastdiv(pooled ? g.Wp : 1); a.dHp = make_fastdiv(pooled ? g.Hp : 1);
        a.upd_words = (int)(((long long)g.S * g.Ho * g.Wo + 63) / 64);
        a.pool_words = pooled ? (int)(((long long)g.S * g.Hp * g.Wp + 63) / 64) : 0;
        a.chg_words = (int)(((long long)g.S * g.H * g.W + 63) / 64);
        a.upd_blocks = (a.upd_words + kCountWords - 1) / kCountWords;
        a.pool_blocks = (a.pool_words + kCountWords - 1) / kCountWords;
        const int grid = a.upd_blocks + a.pool_blocks + (count ? (a.chg_words + kCountWords - 1) / kCountWords : 0);
        // LDS for the largest piece any workgroup reads (at most kRegionWords, or dilate_counts() is
        // false): small pieces leave room for more workgroups per compute unit
        long long rw = dilate_region_words(g, false);
        if (pooled && dilate_region_words(g, true) > rw) rw = dilate_region_words(g, true);
        a.region_words = (int)rw;
        const unsigned lds = (unsigned)(rw + 2) * 8u;
        if (g.chg_bytes)
            launch_kernel(tm, dilate_words_kernel<true>, dim3(grid), dim3(kBlock), lds, st, a);
        else
            launch_kernel(tm, dilate_words_kernel<false>, dim3(grid), dim3(kBlock), lds, st, a);
        return hipGetLastError();
    }
    const int ub = (g.S * g.Ho * g.Wo + kBlock - 1) / kBlock;
    const int pb = pooled ? (g.S * g.Hp * g.Wp + kBlock - 1) / kBlock : 0;
    if (g.chg_bytes)
        launch_kernel(tm, dilate_kernel<true>, dim3(ub + pb), dim3(kBlock), 0, st, chg_bits, upd_bits, pool_bits, g,
                           ub);
    else
        launch_kernel(tm, dilate_kernel<false>, dim3(ub + pb), dim3(kBlock), 0, st, chg_bits, upd_bits, pool_bits, g,
                           ub);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Change-index extraction.  A workgroup owns 256 or 512 bitmap words, one or two consecutive ones
// per thread.  Where its output starts it finds out itself, without waiting for anybody: by adding the
// set-bit counts of all groups of words before its own (left by the dilation kernel or by
// compact_count_kernel; 16-byte loads, at most 32 KiB from L2), or for small maps by counting the
// preceding words.  Ordered and deterministic.  The threads scan the popcounts of their words and
// expand the bits.  A workgroup with at most kCompactStage entries goes through an LDS staging
// buffer, shifted so that LDS index and global address agree modulo 16 bytes -- a word with few
// set bits is walked by its holder, a word with many by the whole wave at once (lane b tests bit
// b and ranks it with a popcount) -- and copies it out with 16-byte stores, every wave writing
// one contiguous kilobyte.  A workgroup with more (a moving object's solid block of set words)
// writes straight to the list: completely set words four per wave step with 16-byte stores, the
// others one per step.
// ------------------------------------------------------------------------------------------
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
// set) is packed on the fly.
__device__ __forceinline__ uint64_t map_word(const CompactJob &job, int i)
{
    if (!job.bytes) return job.bits[i];
    uint64_t w = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) w |= (uint64_t)nonzero_bytes(job.bits[(size_t)i * 8 + k]) << (8 * k);
    return w;
}

// Set bits per group of kCountWords words, for maps with so many words that letting every
// workgroup recount all preceding ones would dominate (see compact_kernel).
__global__ __launch_bounds__(kBlock) void compact_count_kernel(CompactJobs jobs)
{
    const CompactJob job = jobs.j[blockIdx.y];
    const int i = blockIdx.x * kBlock + threadIdx.x; // one word per thread; a wave covers two groups
    if (blockIdx.x * kBlock >= job.nwords) return;
    int c = i < job.nwords ? __popcll(map_word(job, i)) : 0;
#pragma unroll
    for (int d = kCountWords / 2; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
    if ((threadIdx.x & (kCountWords - 1)) == 0 && i < job.nwords) job.group_counts[i / kCountWords] = c;
}

typedef int intx4_a4 __attribute__((ext_vector_type(4), aligned(4))); // four list entries starting at any of them

// WPT words per thread: two for maps of millions of positions (fewer workgroups, fewer counts to
// add up per workgroup), one below that (more workgroups to spread a small map's set words over).
template <bool TWO_LEVEL, int WPT>
__global__ __launch_bounds__(kBlock) void compact_kernel(CompactJobs jobs)
{
    constexpr int kWords = WPT * kBlock; // words per workgroup
    static_assert(WPT == 1 || WPT == 2, "one or two words per thread");
    static_assert(kWords % (4 * kCountWords) == 0, "whole 16-byte loads of group counts");
    __shared__ __align__(16) int stage[kCompactStage + 4];
    __shared__ uint64_t sword[kWords];
    __shared__ int soff[kWords];
    __shared__ int2 sfull[kBlock / 64][WPT * 64]; // per wave: offset and first position of its completely set words
    __shared__ int swave[kBlock / 64];
    __shared__ int swave2[kBlock / 64];
    const CompactJob job = jobs.j[blockIdx.y];
    const int w0 = blockIdx.x * kWords;
    if (w0 >= job.nwords) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // set bits in all words before this workgroup's (the loads go out together with those of the
    // workgroup's own words below: one round trip, not two)
    int before = 0;
    if (TWO_LEVEL) {
        const int4 *g4 = reinterpret_cast<const int4 *>(job.group_counts);
        const int n4 = (int)blockIdx.x * (kWords / kCountWords / 4);
        for (int i = tid; i < n4; i += kBlock) {
            const int4 v = g4[i];
            before += v.x + v.y + v.z + v.w;
        }
    } else {
        for (int i = tid; i < w0; i += kBlock) before += __popcll(map_word(job, i));
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) before += __shfl_xor(before, d, 64);
    if (lane == 0) swave[wave] = before;

    // this workgroup's words: for the scan thread t holds the WPT consecutive words WPT t ... of them
    {
        const int i0 = w0 + WPT * tid;
        uint64_t m0 = 0, m1 = 0;
        if (WPT == 2 && !job.bytes && i0 + 1 < job.nwords) {
            const ulonglong2 v = *reinterpret_cast<const ulonglong2 *>(job.bits + i0);
            m0 = v.x;
            m1 = v.y;
        } else {
            if (i0 < job.nwords) m0 = map_word(job, i0);
            if (WPT == 2 && i0 + 1 < job.nwords) m1 = map_word(job, i0 + 1);
        }
        const int c0 = __popcll(m0), sum = c0 + __popcll(m1);
        const int incl = wave_incl_scan(sum, lane);
        if (lane == 63) swave2[wave] = incl;
        sword[WPT * tid] = m0;
        soff[WPT * tid] = incl - sum;        // still without the waves before this one
        if (WPT == 2) {
            sword[2 * tid + 1] = m1;
            soff[2 * tid + 1] = incl - sum + c0;
        }
    }
    __syncthreads();
    int total = 0, wave_off[kBlock / 64];
#pragma unroll
    for (int i = 0; i < kBlock / 64; ++i) {
        wave_off[i] = total;
        total += swave2[i];
    }
    const bool last = w0 + kWords >= job.nwords;
    if (total == 0 && !last) return; // nothing to write: most workgroups of a quiet scene end here
    int prefix = 0;
#pragma unroll
    for (int i = 0; i < kBlock / 64; ++i) prefix += swave[i];
    // For the expansion the words are dealt out again: lane l of wave v takes word 4 l + v (and
    // 256 + 4 l + v), so that of any run of consecutive words -- a solid block of set words, say --
    // each wave holds a quarter.
    uint64_t m[WPT];
    int c[WPT], o[WPT], pos[WPT];
#pragma unroll
    for (int h = 0; h < WPT; ++h) {
        const int wi = 256 * h + 4 * lane + wave;
        m[h] = sword[wi];
        c[h] = __popcll(m[h]);
        o[h] = soff[wi] + wave_off[wi / (64 * WPT)]; // word wi was scanned by thread wi / WPT
        pos[h] = (w0 + wi) * 64;
    }
    int *dst = job.list + prefix;
    if (total > kCompactStage) {
        // Many entries: straight to the list.  Completely set words -- the inside of a moving object --
        // four at a time: each quarter of the wave writes the 64 consecutive positions of one of them
        // as sixteen 16-byte stores.  Any other word by the whole wave at once: lane b tests bit b, ranks
        // it with a popcount, and the set lanes write consecutive entries.
        const uint64_t below = (1ull << lane) - 1ull;
        int nfull = 0;
#pragma unroll
        for (int h = 0; h < WPT; ++h) {
            const bool full = c[h] == 64;
            const uint64_t fb = __ballot(full);
            if (full) sfull[wave][nfull + __popcll(fb & below)] = make_int2(o[h], pos[h]);
            nfull += __popcll(fb);
            uint64_t todo = __ballot(c[h] > 0 && !full);
            while (todo) {
                const int src = __ffsll((unsigned long long)todo) - 1;
                todo &= todo - 1ull;
                const uint64_t w = ((uint64_t)(unsigned)__builtin_amdgcn_readlane((int)(m[h] >> 32), src) << 32) |
                                   (unsigned)__builtin_amdgcn_readlane((int)m[h], src);
                const int ow = __builtin_amdgcn_readlane(o[h], src), pw = __builtin_amdgcn_readlane(pos[h], src);
                if ((w >> lane) & 1ull) dst[ow + __popcll(w & below)] = pw + lane;
            }
        }
        __builtin_amdgcn_wave_barrier(); // sfull[wave] is written and read by this wave only
        for (int j = lane >> 4; j < nfull; j += 4) {
            const int2 e = sfull[wave][j];
            const int q = 4 * (lane & 15);
            *reinterpret_cast<intx4_a4 *>(dst + e.x + q) = (intx4_a4){e.y + q, e.y + q + 1, e.y + q + 2, e.y + q + 3};
        }
    } else {
        // few: through the staging buffer, shifted so that dst[e] and stage[e + shift] are aligned alike
        const int shift = (int)((reinterpret_cast<uintptr_t>(dst) >> 2) & 3);
#pragma unroll
        for (int h = 0; h < WPT; ++h) {
            if (c[h] > 0 && c[h] <= kCompactDense) { // a word with few set bits: its holder walks them
                int e = o[h] + shift;
                uint64_t r = m[h];
                while (r) {
                    stage[e++] = pos[h] + __ffsll((unsigned long long)r) - 1;
                    r &= r - 1ull;
                }
            }
            uint64_t todo = __ballot(c[h] > kCompactDense); // one with many: the whole wave, one step
            while (todo) {
                const int src = __ffsll((unsigned long long)todo) - 1;
                todo &= todo - 1ull;
                const uint64_t w = ((uint64_t)(unsigned)__builtin_amdgcn_readlane((int)(m[h] >> 32), src) << 32) |
                                   (unsigned)__builtin_amdgcn_readlane((int)m[h], src);
                const int ow = __builtin_amdgcn_readlane(o[h], src), pw = __builtin_amdgcn_readlane(pos[h], src);
                if ((w >> lane) & 1ull) stage[ow + shift + __popcll(w & ((1ull << lane) - 1ull))] = pw + lane;
            }
        }
        __syncthreads();
        int head = (4 - shift) & 3; // entries before the first 16-byte boundary of dst
        if (head > total) head = total;
        if (tid < head) dst[tid] = stage[tid + shift];
        const int body = (total - head) >> 2;
        const int4 *s4 = reinterpret_cast<const int4 *>(stage + head + shift); // a multiple of four ints (or body == 0)
        int4 *d4 = reinterpret_cast<int4 *>(dst + head);
        for (int j = tid; j < body; j += kBlock) d4[j] = s4[j];
        const int done = head + 4 * body;
        if (tid < total - done) dst[done + tid] = stage[done + tid + shift];
    }
    if (tid == 0 && last) *job.count = prefix + total;
}

bool compact_two_level(int nwords) { return nwords > 6144; }

// a multiple of 16 bytes, so that the arrays of a layer's three maps, one behind the other, all
// start on a 16-byte boundary
size_t compact_group_count_bytes(int nwords) { return (((size_t)nwords / kCountWords + 8 + 3) & ~(size_t)3) * sizeof(int); }

hipError_t compact(hipStream_t st, const CompactJob *jobs, int njobs, bool groups_ready, const Timing &tm)
{
    if (njobs < 1 || njobs > 3) return hipErrorInvalidValue;
    CompactJobs js;
    int maxw = 1;
    for (int i = 0; i < 3; ++i) {
        js.j[i] = jobs[i < njobs ? i : 0];
        if (i < njobs && jobs[i].nwords > maxw) maxw = jobs[i].nwords;
    }
    for (int i = 0; i < njobs; ++i) // 16-byte loads of word pairs
        if (!jobs[i].bits || reinterpret_cast<uintptr_t>(jobs[i].bits) % 16 || !jobs[i].list || !jobs[i].count) return hipErrorInvalidValue;
    const bool two = maxw > kCompactTwoWordsFrom; // words per thread
    const int gx = (maxw + (two ? 2 : 1) * kBlock - 1) / ((two ? 2 : 1) * kBlock);
    // a byte map costs eight loads per word: letting every workgroup recount all preceding words is
    // worth it for much smaller maps only
    bool any_bytes = false;
    for (int i = 0; i < njobs; ++i) any_bytes = any_bytes || jobs[i].bytes != 0;
    if (groups_ready || compact_two_level(maxw) || (any_bytes && maxw > kCompactTwoLevelBytesFrom)) {
        for (int i = 0; i < njobs; ++i)
            if (!jobs[i].group_counts || reinterpret_cast<uintptr_t>(jobs[i].group_counts) % 16) return hipErrorInvalidValue;
        Timing t2 = tm;
        if (!groups_ready) {
            launch_kernel(Timing{tm.start, nullptr}, compact_count_kernel, dim3((maxw + kBlock - 1) / kBlock, njobs), dim3(kBlock), 0, st, js);
            t2 = Timing{nullptr, tm.stop};
        }
        if (two)
            launch_kernel(t2, compact_kernel<true, 2>, dim3(gx, njobs), dim3(kBlock), 0, st, js);
        else
            launch_kernel(t2, compact_kernel<true, 1>, dim3(gx, njobs), dim3(kBlock), 0, st, js);
    } else {
        launch_kernel(tm, compact_kernel<false, 1>, dim3(gx, njobs), dim3(kBlock), 0, st, js);
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
// Geometry of a pooling launch; the divisors are the invariant ones of its index arithmetic
// (integer division is emulated on this hardware, and these kernels are short).
struct PoolGeom {
    int V, k, Wo, No, Wp, Np;
    FastDiv dV, dNp, dWp;
};
static PoolGeom pool_geom(int V, int k, int Wo, int No, int Wp, int Np)
{
    return {V, k, Wo, No, Wp, Np, make_fastdiv(V), make_fastdiv(Np), make_fastdiv(Wp)};
}

template <int DT>
__device__ __forceinline__ void pool_unit(bool active, int g, int v, const uint4 *__restrict__ in,
                                          uint4 *__restrict__ pooled, const PoolGeom &pg,
                                          unsigned char *__restrict__ next_flags, float next_tau, int next_force)
{
    const int V = pg.V, k = pg.k, Wo = pg.Wo, No = pg.No, Wp = pg.Wp, Np = pg.Np;
    const int lane = threadIdx.x & 63;
    const bool pow2 = (V & (V - 1)) == 0 && V <= 64;
    uint4 m = make_uint4(0u, 0u, 0u, 0u);
    bool f = false;
    if (active) {
        const int st = fast_div(g, pg.dNp), pp = g - st * Np;
        const int py = fast_div(pp, pg.dWp), px = pp - py * Wp;
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

// The 2 x 2 window, kPoolBatch items per thread: the list entries (or map bits) of all items are
// fetched first, then all window values (and the values about to be replaced), so that a thread
// has up to 4 * kPoolBatch 16-byte loads in flight instead of one dependent round trip after the
// other -- on maps of millions of positions the kernel is bound by exactly that latency.
static constexpr int kPoolBatch = 4;

template <int DT>
__device__ __forceinline__ void pool_batch_2x2(const bool (&active)[kPoolBatch], const int (&g)[kPoolBatch],
                                               const int (&v)[kPoolBatch], const uint4 *__restrict__ in,
                                               uint4 *__restrict__ pooled, const PoolGeom &pg,
                                               unsigned char *__restrict__ next_flags, float next_tau, int next_force)
{
    const int V = pg.V, lane = threadIdx.x & 63;
    const bool pow2 = (V & (V - 1)) == 0 && V <= 64;
    const bool compare = next_flags != nullptr && !next_force;
    uint4 w[kPoolBatch][4], old[kPoolBatch];
#pragma unroll
    for (int k = 0; k < kPoolBatch; ++k) {
        if (!active[k]) continue;
        const int st = fast_div(g[k], pg.dNp), pp = g[k] - st * pg.Np;
        const int py = fast_div(pp, pg.dWp), px = pp - py * pg.Wp;
        const long long base = ((long long)st * pg.No + (long long)(py * 2) * pg.Wo + px * 2) * V + v[k];
        w[k][0] = in[base];
        w[k][1] = in[base + V];
        w[k][2] = in[base + (long long)pg.Wo * V];
        w[k][3] = in[base + (long long)pg.Wo * V + V];
        if (compare) old[k] = pooled[(long long)g[k] * V + v[k]];
    }
#pragma unroll
    for (int k = 0; k < kPoolBatch; ++k) {
        uint4 m = make_uint4(0u, 0u, 0u, 0u);
        bool f = false;
        if (active[k]) {
            m = unit_max<DT>(unit_max<DT>(w[k][0], w[k][1]), unit_max<DT>(w[k][2], w[k][3]));
            // change detection of the layer this map feeds: new value against the one it replaces
            if (next_flags) f = next_force != 0 || unit_exceeds<DT>(m, old[k], next_tau);
        }
        if (next_flags) {
            if (pow2) { // the V lanes of a position sit next to each other in the wave
                const unsigned long long B = __ballot(f);
                const unsigned long long grp = (V == 64) ? ~0ull : (((1ull << V) - 1ull) << (lane & ~(V - 1)));
                if (active[k] && v[k] == 0 && (B & grp) != 0ull) next_flags[g[k]] = 1;
            } else if (f) {
                next_flags[g[k]] = 1;
            }
        }
        if (active[k]) pooled[(long long)g[k] * V + v[k]] = m;
    }
}

template <int DT>
__global__ __launch_bounds__(kBlock) void pool_sparse_kernel(const int *__restrict__ list,
                                                             const int *__restrict__ count,
                                                             const uint4 *__restrict__ in,
                                                             uint4 *__restrict__ pooled, PoolGeom pg,
                                                             unsigned char *__restrict__ next_flags,
                                                             float next_tau, int next_force)
{
    const int total = *count * pg.V; // units: below 2^30 (checked by the host)
    const int step = (int)gridDim.x * kBlock;
    // whole waves iterate together (the last round with some lanes inactive)
    if (pg.k == 2) {
        for (int i0 = (int)blockIdx.x * kBlock; i0 < total; i0 += kPoolBatch * step) {
            bool active[kPoolBatch];
            int g[kPoolBatch], v[kPoolBatch];
#pragma unroll
            for (int k = 0; k < kPoolBatch; ++k) {
                const long long idx = (long long)i0 + (long long)k * step + (int)threadIdx.x;
                active[k] = idx < total;
                const int u = active[k] ? fast_div((int)idx, pg.dV) : 0;
                v[k] = active[k] ? (int)idx - u * pg.V : 0;
                g[k] = active[k] ? list[u] : 0;
            }
            pool_batch_2x2<DT>(active, g, v, in, pooled, pg, next_flags, next_tau, next_force);
        }
        return;
    }
    for (int i0 = (int)blockIdx.x * kBlock; i0 < total; i0 += step) {
        const int idx = i0 + (int)threadIdx.x;
        const bool active = idx < total;
        const int u = active ? fast_div(idx, pg.dV) : 0, v = active ? idx - u * pg.V : 0;
        const int g = active ? list[u] : 0;
        pool_unit<DT>(active, g, v, in, pooled, pg, next_flags, next_tau, next_force);
    }
}

// Whether pooled position g is to be recomputed according to the bitmap (over the pooled positions,
// or from_outputs: over the convolution outputs, any of the k x k under g).
__device__ __forceinline__ bool pool_bit(const uint64_t *__restrict__ bits, int from_outputs, int g, const PoolGeom &pg)
{
    if (!from_outputs) return ((bits[g >> 6] >> (g & 63)) & 1ull) != 0ull;
    const int st = fast_div(g, pg.dNp), pp = g - st * pg.Np;
    const int py = fast_div(pp, pg.dWp), px = pp - py * pg.Wp;
    bool any = false;
    for (int j = 0; j < pg.k; ++j) {
        const int q0 = st * pg.No + (py * pg.k + j) * pg.Wo + px * pg.k;
        for (int i = 0; i < pg.k; ++i) any |= ((bits[(q0 + i) >> 6] >> ((q0 + i) & 63)) & 1ull) != 0ull;
    }
    return any;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void pool_masked_kernel(const uint64_t *__restrict__ bits, int from_outputs,
                                                             int total_px,
                                                             const uint4 *__restrict__ in,
                                                             uint4 *__restrict__ pooled, PoolGeom pg,
                                                             unsigned char *__restrict__ next_flags,
                                                             float next_tau, int next_force)
{
    const int total = total_px * pg.V;
    const int step = (int)gridDim.x * kBlock;
    if (pg.k == 2) {
        for (int i0 = (int)blockIdx.x * kBlock; i0 < total; i0 += kPoolBatch * step) {
            bool active[kPoolBatch];
            int g[kPoolBatch], v[kPoolBatch];
#pragma unroll
            for (int k = 0; k < kPoolBatch; ++k) {
                const long long idx = (long long)i0 + (long long)k * step + (int)threadIdx.x;
                const bool in_range = idx < total;
                g[k] = in_range ? fast_div((int)idx, pg.dV) : 0;
                v[k] = in_range ? (int)idx - g[k] * pg.V : 0;
                active[k] = in_range && pool_bit(bits, from_outputs, g[k], pg);
            }
            pool_batch_2x2<DT>(active, g, v, in, pooled, pg, next_flags, next_tau, next_force);
        }
        return;
    }
    for (int i0 = (int)blockIdx.x * kBlock; i0 < total; i0 += step) {
        const int idx = i0 + (int)threadIdx.x;
        bool active = idx < total;
        const int g = active ? fast_div(idx, pg.dV) : 0, v = active ? idx - g * pg.V : 0;
        if (active) active = pool_bit(bits, from_outputs, g, pg);
        pool_unit<DT>(active, g, v, in, pooled, pg, next_flags, next_tau, next_force);
    }
}

hipError_t pool_sparse(hipStream_t st, const int *list, const int *count, int max_count, const void *in,
                       void *pooled, int V, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force, int dtype, const Timing &tm)
{
    long long work = (long long)max_count * V;
    if (work >= (1ll << 30) || V < 1 || Np < 1 || Wp < 1) return hipErrorInvalidValue; // 32-bit indices, with room for the grid stride
    const PoolGeom pg = pool_geom(V, k, Wo, No, Wp, Np);
    const int per_thread = k == 2 ? kPoolBatch : 1;
    long long grid = (work + (long long)kBlock * per_thread - 1) / ((long long)kBlock * per_thread);
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    const uint4 *i4 = static_cast<const uint4 *>(in);
    uint4 *p4 = static_cast<uint4 *>(pooled);
    if (dtype == kBF16)
        launch_kernel(tm, pool_sparse_kernel<kBF16>, dim3((int)grid), dim3(kBlock), 0, st, list, count, i4, p4, pg,
                      next_flags, next_tau, next_force);
    else
        launch_kernel(tm, pool_sparse_kernel<kF32>, dim3((int)grid), dim3(kBlock), 0, st, list, count, i4, p4, pg,
                      next_flags, next_tau, next_force);
    return hipGetLastError();
}

hipError_t pool_masked(hipStream_t st, const uint64_t *bits, int from_outputs, int total, const void *in,
                       void *pooled, int V, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force, int dtype, const Timing &tm)
{
    long long work = (long long)total * V;
    if (work >= (1ll << 30) || V < 1 || Np < 1 || Wp < 1) return hipErrorInvalidValue; // 32-bit indices, with room for the grid stride
    const PoolGeom pg = pool_geom(V, k, Wo, No, Wp, Np);
    const int per_thread = k == 2 ? kPoolBatch : 1;
    long long grid = (work + (long long)kBlock * per_thread - 1) / ((long long)kBlock * per_thread);
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    const uint4 *i4 = static_cast<const uint4 *>(in);
    uint4 *p4 = static_cast<uint4 *>(pooled);
    if (dtype == kBF16)
        launch_kernel(tm, pool_masked_kernel<kBF16>, dim3((int)grid), dim3(kBlock), 0, st, bits, from_outputs, total, i4, p4,
                      pg, next_flags, next_tau, next_force);
    else
        launch_kernel(tm, pool_masked_kernel<kF32>, dim3((int)grid), dim3(kBlock), 0, st, bits, from_outputs, total, i4, p4,
                      pg, next_flags, next_tau, next_force);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Stored map [S*No][V units] -> planar float32 [S][M][No].  Consecutive lanes take consecutive
// pixels' units (16-byte reads) and write one contiguous run per channel plane.
// ------------------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kBlock) void map_to_planar_kernel(const uint4 *__restrict__ map,
                                                               float *__restrict__ planar, int M, int V,
                                                               int No, int total, FastDiv dNo, FastDiv dV)
{
    constexpr int E = Unit<DT>::N;
    for (int idx = (int)blockIdx.x * kBlock + (int)threadIdx.x; idx < total; idx += (int)gridDim.x * kBlock) {
        const int sv = fast_div(idx, dNo), q = idx - sv * No;
        const int st = fast_div(sv, dV), v = sv - st * V;
        const uint4 a = map[(size_t)(st * No + q) * V + v];
        float *dst = planar + ((size_t)st * M + (size_t)E * v) * No + q;
#pragma unroll
        for (int i = 0; i < E; ++i)
            if (E * v + i < M) dst[(size_t)i * No] = Unit<DT>::get(a, i);
    }
}

// The same for maps of at most kPlanarUnits units per pixel: a thread takes a whole pixel, so that
// a wave reads one contiguous run of the map (with a thread per unit each load instruction would
// touch every V-th unit only and leave the rest of every line to a later instruction).
static constexpr int kPlanarUnits = 4;

template <int DT, int V>
__global__ __launch_bounds__(kBlock) void map_to_planar_pixel_kernel(const uint4 *__restrict__ map,
                                                                     float *__restrict__ planar, int M, int No,
                                                                     int total_px, FastDiv dNo)
{
    constexpr int E = Unit<DT>::N;
    for (int g = (int)blockIdx.x * kBlock + (int)threadIdx.x; g < total_px; g += (int)gridDim.x * kBlock) {
        const int st = fast_div(g, dNo), q = g - st * No;
        uint4 a[V];
#pragma unroll
        for (int v = 0; v < V; ++v) a[v] = map[(size_t)g * V + v];
        float *dst = planar + (size_t)st * M * No + q;
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int i = 0; i < E; ++i)
                if (E * v + i < M) dst[(size_t)(E * v + i) * No] = Unit<DT>::get(a[v], i);
    }
}

hipError_t map_to_planar(hipStream_t st, const void *map, float *planar, int M, int V, int No, int S, int dtype,
                         const Timing &tm)
{
    const long long total = (long long)S * V * No; // units of the map
    if (total >= (1ll << 30) || V < 1 || No < 1) return hipErrorInvalidValue; // 32-bit indices, with room for the grid stride
    const uint4 *m4 = static_cast<const uint4 *>(map);
    const FastDiv dNo = make_fastdiv(No), dV = make_fastdiv(V);
    if (V <= kPlanarUnits) {
        const int px = S * No;
        int grid = (px + kBlock - 1) / kBlock;
        if (grid > 16384) grid = 16384;
#define CBK_LAUNCH(DT_, V_)                                                                                            \
    launch_kernel(tm, map_to_planar_pixel_kernel<DT_, V_>, dim3(grid), dim3(kBlock), 0, st, m4, planar, M, No, px, dNo)
#define CBK_BY_V(DT_)                                                                                                  \
    switch (V) {                                                                                                       \
    case 1: CBK_LAUNCH(DT_, 1); break;                                                                                 \
    case 2: CBK_LAUNCH(DT_, 2); break;                                                                                 \
    case 3: CBK_LAUNCH(DT_, 3); break;                                                                                 \
    default: CBK_LAUNCH(DT_, 4); break;                                                                                \
    }
        if (dtype == kBF16) {
            CBK_BY_V(kBF16)
        } else {
            CBK_BY_V(kF32)
        }
#undef CBK_BY_V
#undef CBK_LAUNCH
        return hipGetLastError();
    }
    long long grid = (total + kBlock - 1) / kBlock;
    if (grid > 8192) grid = 8192;
    if (grid < 1) grid = 1;
    if (dtype == kBF16)
        launch_kernel(tm, map_to_planar_kernel<kBF16>, dim3((int)grid), dim3(kBlock), 0, st, m4, planar, M, V, No,
                      (int)total, dNo, dV);
    else
        launch_kernel(tm, map_to_planar_kernel<kF32>, dim3((int)grid), dim3(kBlock), 0, st, m4, planar, M, V, No,
                      (int)total, dNo, dV);
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
