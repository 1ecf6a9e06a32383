// Host-side launch interface of the gfx950 kernels.  Everything here enqueues work on the
// given stream and returns the hipError_t of the launch; nothing synchronises or allocates.
//
// Internal data layout (all device memory):
//   maps      [stream][y][x][Cs], channel-contiguous, float32 or bfloat16; Cs = channels rounded
//             up to a whole number of 16-byte units (4 floats / 8 bfloat16), padding channels are
//             zero.  Sizes are passed in units: V = units per pixel.  "pixel g" = stream*H*W + y*W + x.
//   bitmaps   one bit per pixel g, packed in uint64 words (bit g%64 of word g/64);
//             bits at or beyond the pixel count are zero.
//   lists     int32 pixel indices g, ascending, with their length in an int32 counter.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace cbk {

// Optional pair of events that receive a launch's own start and end time stamps (the kernel's
// execution interval as the device records it, without the gaps before and after that events
// recorded on the stream around a launch would include).  Both null: an ordinary launch.
struct Timing {
    hipEvent_t start = nullptr, stop = nullptr;
};

template <typename F, typename... Args>
inline void launch_kernel(const Timing &tm, F kernel, dim3 grid, dim3 block, unsigned smem, hipStream_t st, Args... args)
{
    if (tm.start || tm.stop)
        hipExtLaunchKernelGGL(kernel, grid, block, smem, st, tm.start, tm.stop, 0u, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, smem, st, args...);
}

enum { kF32 = 0, kBF16 = 1 }; // storage type of maps and filter matrices (accumulation is float32)
inline int elems_per_unit(int dt) { return dt == kBF16 ? 8 : 4; }
inline int elem_bytes(int dt) { return dt == kBF16 ? 2 : 4; }

// float -> bfloat16 bits, round to nearest even; NaN stays a (quiet) NaN.
__host__ __device__ inline unsigned short bf16_bits(float f)
{
    union { float f; unsigned int u; } c;
    c.f = f;
    unsigned int u = c.u;
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__host__ __device__ inline float bf16_value(unsigned short b)
{
    union { float f; unsigned int u; } c;
    c.u = (unsigned int)b << 16;
    return c.f;
}

// One 16-byte unit of a map: 4 floats or 8 bfloat16.
template <int DT>
struct Unit;
template <>
struct Unit<kF32> {
    static constexpr int N = 4;
    static __device__ __forceinline__ float get(const uint4 &u, int i) { return __uint_as_float((&u.x)[i]); }
    static __device__ __forceinline__ void set(uint4 &u, int i, float f) { (&u.x)[i] = __float_as_uint(f); }
};
template <>
struct Unit<kBF16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ float get(const uint4 &u, int i)
    {
        const unsigned int w = (&u.x)[i >> 1];
        return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    static __device__ __forceinline__ void set(uint4 &u, int i, float f) // rounds to bfloat16
    {
        const unsigned int b = bf16_bits(f);
        unsigned int &w = (&u.x)[i >> 1];
        w = (i & 1) ? ((w & 0x0000ffffu) | (b << 16)) : ((w & 0xffff0000u) | b);
    }
};

// Change test on one unit: one subtraction, one absolute value and one strict comparison per
// channel, in float (Section 3.1); a NaN difference compares false and does not flag.
template <int DT>
__device__ __forceinline__ bool unit_exceeds(const uint4 &a, const uint4 &r, const float tau)
{
    bool f = false;
#pragma unroll
    for (int i = 0; i < Unit<DT>::N; ++i) f = f || (fabsf(Unit<DT>::get(a, i) - Unit<DT>::get(r, i)) > tau);
    return f;
}

template <int DT>
__device__ __forceinline__ uint4 unit_max(const uint4 &a, const uint4 &b)
{
    uint4 m = a;
#pragma unroll
    for (int i = 0; i < Unit<DT>::N; ++i) Unit<DT>::set(m, i, fmaxf(Unit<DT>::get(a, i), Unit<DT>::get(b, i)));
    return m;
}

// ---- change detection (Section 3.1, first formula) ---------------------------------------
// Planar float32 frame [S][C][N] against the stored previous input kept as a map of V units per
// pixel (bfloat16 storage: the frame is rounded to bfloat16 first and compared as such).
// Writes the change bitmap; refreshes the stored input (hold == 0: everywhere;
// hold == 1: `cur` receives the frame as a map and `ref` is refreshed only where flagged).
// force != 0: every pixel is flagged and ref is not read (first frame / dense mode).
// clear_words 64-bit words starting at clear are zeroed by the same launch (the byte change maps
// that later kernels of the frame fill in); they must not overlap bits.
// packed != 0 (only where detect_frame_packs(dtype, C, S * N)): the stored map holds C float32 values
// per pixel and no padding channels.
bool detect_frame_packs(int dtype, int C, long long pixels);
hipError_t detect_frame(hipStream_t st, const float *frame, void *ref, void *cur, uint64_t *bits, int C, int V,
                        int N, int S, float tau, int hold, int force, int dtype, int packed, uint64_t *clear,
                        long long clear_words, const Timing &tm = Timing());

// Map against map (layers fed by a stored output map).  x and ref are [S*N][V units].
hipError_t detect_map(hipStream_t st, const void *x, void *ref, uint64_t *bits, int V, int total, float tau,
                      int hold, int force, int dtype, const Timing &tm = Timing());

// Division of a non-negative 32-bit number by an invariant divisor through one 64-bit
// multiplication (integer division is emulated with dozens of instructions on this hardware).
// Exact for 0 <= n < 2^31 and 1 <= d < 2^31: with l = ceil(log2 d) and m = floor(2^(31+l) / d) + 1,
// m*d - 2^(31+l) lies in (0, d], which keeps floor(n*m / 2^(31+l)) equal to floor(n / d).
struct FastDiv {
    unsigned m;
    int shift;
    int d;
};
inline FastDiv make_fastdiv(int d)
{
    int l = 0;
    while ((1ll << l) < d) ++l;
    FastDiv f;
    f.d = d;
    f.shift = 31 + l;
    f.m = (unsigned)(((1ull << (31 + l)) / (unsigned long long)d) + 1ull);
    return f;
}
__host__ __device__ inline int fast_div(int n, const FastDiv &f)
{
    return (int)(((unsigned long long)(unsigned)n * f.m) >> f.shift);
}

// ---- dilation by the filter support (Section 3.1, second formula) -------------------------
// upd bit (stream, qy, qx) = OR of the change bits inside that output's receptive field.
// If pool_bits != nullptr also writes, for a k x k / stride k pooling that follows, the
// bitmap of pooled positions whose window contains an updated output.
struct DilateGeom {
    int S, H, W, Ho, Wo, kh, kw, stride, pad; // convolution geometry
    int pool_k, Hp, Wp;                       // pooling that follows (pool_k == 0: none)
    int chg_bytes;                            // the change map has one byte per pixel instead of one bit
};
// groups: null, or one array of compact_group_count_bytes() bytes per map (update map, pooled map,
// change map, in this order; the pooled one may be null without pooling).  When dilate_counts(g)
// -- a geometry the word-at-a-time kernel handles -- the launch also fills them with the number of
// set bits per group of words, which compact() then need not count (groups_ready).
struct DilateGroups {
    int *upd, *pool, *chg;
};
bool dilate_counts(const DilateGeom &g);
hipError_t dilate(hipStream_t st, const uint64_t *chg_bits, uint64_t *upd_bits, uint64_t *pool_bits,
                  const DilateGeom &g, const DilateGroups *groups = nullptr, const Timing &tm = Timing());

// ---- change-index extraction (Section 3.1) -------------------------------------------------
// Up to three bitmaps -> ascending index lists and counts in one launch.
struct CompactJob {
    const uint64_t *bits; // bitmap, or (bytes != 0) a map with one byte per pixel, padded to 64 pixels
    int bytes;
    int nwords;           // 64-pixel words
    int *list;
    int *count;
    int *group_counts;    // scratch of compact_group_count_bytes(nwords) bytes; needed (non-null) when
                          // compact_two_level(nwords), i.e. for maps of several hundred thousand pixels
};
bool compact_two_level(int nwords);
size_t compact_group_count_bytes(int nwords);
// groups_ready: every job's group_counts already holds the set bits of its groups of words.
hipError_t compact(hipStream_t st, const CompactJob *jobs, int njobs, bool groups_ready = false,
                   const Timing &tm = Timing());


// ---- gathered matrix generation + multiplication + output update (Section 3.1) -------------
struct GemmArgs {
    int dtype;          // kF32 or kBF16: storage of x, wt and out
    const void *x;      // input map, pix_words 4-byte words per pixel, followed by at least 16 bytes of zeros
    const void *wt;     // filter matrix, [Mpad][Kpad], k = (j*kw + i)*Cs + c, zero padded
    const float *bias;  // [Mpad] float32
    const int2 *taps;   // one entry per 16-byte unit of a filter-matrix row:
                        //   .x = offset of that unit, in 4-byte words, from the window origin in the input map,
                        //   .y = j | i << 8 | valid << 16
    const int *list;    // output pixels to recompute
    const int *count;   // their number (device)
    // Alternative to list/count for maps of at most gemm_select_max_words() words: the map of
    // outputs to recompute itself (bit g of word g/64, or one byte per pixel when sel_bytes != 0,
    // padded to whole words).  Every workgroup then ranks the set positions itself and picks those
    // of its tile, which saves the separate extraction launch.  sel_words == 0: use list/count.
    const uint64_t *sel_map;
    int sel_bytes;
    int sel_words;
    // sel_dilate != 0 (stride 1, kw <= 16, change map and the S*H*Wo intermediate map of at most
    // gemm_select_max_words() words each): sel_map is the layer's *change* map over its
    // sel_in_words * 64 input positions, and the kernel derives the outputs to recompute itself
    // by dilating it with the kh x kw filter support (Section 3.1, second formula); workgroup 0
    // writes the resulting bitmap (sel_words words) to upd_out.
    int sel_dilate;
    int sel_in_words;
    uint64_t *upd_out;
    int kh, kw, S;      // filter size; number of streams (used by sel_dilate only)
    void *out;          // stored output map [S*No][Ms]
    int N, H, W, No, Wo, stride, pad;
    FastDiv dNo, dWo, dHo, dNk, dGrid; // by No, Wo, No / Wo, Kpad / gemm_k_multiple(dtype) and grid (gemm_set_divisors)
    FastDiv dVin, dKw;  // by the 16-byte units per filter tap, (pix_words + 3) / 4, and by kw
    int pix_words;      // 4-byte words per input pixel: a multiple of four (whole 16-byte units), or the channel
                        // count of a float32 map stored without padding (units then start at any word and
                        // run into the next pixel's channels, which meet zero filter weights)
    int zero_word;      // word index, relative to x, of 16 bytes of zeros (gathers outside the image read them)
    int Kpad;           // filter-matrix row length in elements, a multiple of gemm_k_multiple(dtype)
    int M, Mpad, Ms, relu;
    int max_pixels;     // upper bound of *count
    float *partial;     // scratch for partial accumulators, gemm_partial_bytes(M, grid) bytes
    int *tickets;       // gemm_ticket_bytes(grid) bytes, zero before the first launch (each launch
                        // leaves them zero again)
    int grid;           // workgroups to launch, from gemm_grid()
    // Change detection of the next layer fused into the output update (used when that layer's
    // stored previous input is this layer's stored output): positions whose new value differs
    // from the replaced one by more than next_tau get their byte set in next_flags (one byte per
    // pixel, zeroed at the start of the frame; several workgroups may store the same 1, no atomics
    // needed).
    unsigned char *next_flags; // nullptr: off
    float next_tau;
    int next_force;            // flag every recomputed position (first frame)
};
int gemm_channel_tile(int M);   // channel tile BM used for M output channels (Mpad = M rounded up to it)
int gemm_k_multiple(int dtype); // Kpad must be a multiple of this many elements (128 bytes)
int gemm_grid(const GemmArgs &a, int compute_units); // needs M, Mpad, Kpad, max_pixels
int gemm_select_max_words(void);
size_t gemm_partial_bytes(int M, int grid);
size_t gemm_ticket_bytes(int grid);
hipError_t gemm_prepare(void);  // one-time function attributes (dynamic LDS size)
void gemm_set_divisors(GemmArgs &a); // fills dNo ... dGrid from No, Wo, Kpad, dtype and grid
// Matrix generation, multiplication and output update (bias, activation, scatter) in one launch.
hipError_t gemm_gather(hipStream_t st, const GemmArgs &a, const Timing &tm = Timing());

// ---- max-pooling at listed pooled positions -----------------------------------------------
// next_flags != nullptr: the pooled map feeds a convolution layer whose stored previous input is
// this very map; compare each recomputed value with the one it replaces against next_tau and set
// the position's byte in that layer's change map (one byte per pixel, zeroed at the start of the frame).
// next_force != 0: flag every recomputed position (first frame).
hipError_t pool_sparse(hipStream_t st, const int *list, const int *count, int max_count, const void *in,
                       void *pooled, int V, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force, int dtype, const Timing &tm = Timing());
// The same at the positions whose bit is set in a bitmap over the total pooled positions (no list);
// from_outputs != 0: the bitmap is over the convolution outputs instead, and a pooled position is
// recomputed if any output in its k x k window is set.
hipError_t pool_masked(hipStream_t st, const uint64_t *bits, int from_outputs, int total, const void *in,
                       void *pooled, int V, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force, int dtype, const Timing &tm = Timing());

// ---- stored map -> caller's planar output --------------------------------------------------
hipError_t map_to_planar(hipStream_t st, const void *map, float *planar, int M, int V, int No, int S, int dtype,
                         const Timing &tm = Timing());

// helpers
hipError_t fill_iota(hipStream_t st, int *list, int n);

} // namespace cbk
