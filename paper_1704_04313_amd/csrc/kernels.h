// Host-side launch interface of the gfx950 kernels.  Everything here enqueues work on the
// given stream and returns the hipError_t of the launch; nothing synchronises or allocates.
//
// Internal data layout (all device memory):
//   maps      [stream][y][x][Cs]  float32, channel-contiguous, Cs = channels rounded up to 4;
//             the padding channels are zero.  "pixel g" = stream*H*W + y*W + x.
//   bitmaps   one bit per pixel g, packed in uint64 words (bit g%64 of word g/64);
//             bits at or beyond the pixel count are zero.
//   lists     int32 pixel indices g, ascending, with their length in an int32 counter.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cbk {

// One subtraction, one absolute value and one strict comparison per channel (Section 3.1);
// a NaN difference compares false and does not flag.
__device__ __forceinline__ bool exceeds(const float4 a, const float4 r, const float tau)
{
    return (fabsf(a.x - r.x) > tau) || (fabsf(a.y - r.y) > tau) || (fabsf(a.z - r.z) > tau) ||
           (fabsf(a.w - r.w) > tau);
}

// ---- change detection (Section 3.1, first formula) ---------------------------------------
// Planar float32 frame [S][C][N] against the stored previous input kept as a map.
// Writes the change bitmap; refreshes the stored input (hold == 0: everywhere;
// hold == 1: `cur` receives the frame as a map and `ref` is refreshed only where flagged).
// force != 0: every pixel is flagged and ref is not read (first frame / dense mode).
hipError_t detect_frame(hipStream_t st, const float *frame, float *ref, float *cur, uint64_t *bits,
                        int C, int Cs, int N, int S, float tau, int hold, int force);

// Map against map (layers fed by a stored output map).  x and ref are [S*N][Cs].
hipError_t detect_map(hipStream_t st, const float *x, float *ref, uint64_t *bits, int Cs, int total,
                      float tau, int hold, int force);

// ---- dilation by the filter support (Section 3.1, second formula) -------------------------
// upd bit (stream, qy, qx) = OR of the change bits inside that output's receptive field.
// If pool_bits != nullptr also writes, for a k x k / stride k pooling that follows, the
// bitmap of pooled positions whose window contains an updated output.
struct DilateGeom {
    int S, H, W, Ho, Wo, kh, kw, stride, pad; // convolution geometry
    int pool_k, Hp, Wp;                       // pooling that follows (pool_k == 0: none)
    int chg_bytes;                            // the change map has one byte per pixel instead of one bit
};
hipError_t dilate(hipStream_t st, const uint64_t *chg_bits, uint64_t *upd_bits, uint64_t *pool_bits,
                  const DilateGeom &g);

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
hipError_t compact(hipStream_t st, const CompactJob *jobs, int njobs);

// ---- gathered matrix generation + multiplication + output update (Section 3.1) -------------
struct GemmArgs {
    const float *x;     // input map [S*N][Cs]
    const float *wt;    // filter matrix, [Mpad][Kpad], k = (j*kw + i)*Cs + c, zero padded
    const float *bias;  // [Mpad]
    const int2 *taps;   // [Kpad/4]: .x = element offset of the tap from the window origin,
                        //           .y = j | i << 8 | valid << 16
    const int *list;    // output pixels to recompute
    const int *count;   // their number (device)
    float *out;         // stored output map [S*No][Ms]
    int N, H, W, No, Wo, stride, pad, Cs, Kpad, M, Mpad, Ms, relu;
    int max_pixels;     // upper bound of *count
    float *partial;     // scratch for partial accumulators, gemm_partial_bytes(M, grid) bytes
    int *tickets;       // gemm_ticket_bytes(grid) bytes, zero before the first launch (each launch
                        // leaves them zero again)
    int grid;           // workgroups to launch, from gemm_grid()
    // Change detection of the next layer fused into the output update (used when that layer's
    // stored previous input is this layer's stored output): positions whose new value differs
    // from the replaced one by more than next_tau get their byte set in next_flags (one byte per
    // pixel, zero on entry; several workgroups may store the same 1, no atomics needed).
    unsigned char *next_flags; // nullptr: off
    float next_tau;
    int next_force;            // flag every recomputed position (first frame)
    // Map this launch clears for the next frame (this layer's own change map, already
    // condensed into lists when the multiplication runs); nullptr: none.
    uint64_t *clear_bits;
    int clear_words;
#ifdef CBK_TRACE
    unsigned long long *trace; // timing study builds only: [grid][2 roles][16] timestamps
#endif
};
int gemm_channel_tile(int M);   // channel tile BM used for M output channels (Mpad = M rounded up to it)
int gemm_k_multiple(void);      // Kpad must be a multiple of this
int gemm_grid(const GemmArgs &a, int compute_units); // needs M, Mpad, Kpad, max_pixels
size_t gemm_partial_bytes(int M, int grid);
size_t gemm_ticket_bytes(int grid);
hipError_t gemm_prepare(void);  // one-time function attributes (dynamic LDS size)
// Matrix generation, multiplication and output update (bias, activation, scatter) in one launch.
hipError_t gemm_gather(hipStream_t st, const GemmArgs &a);

// ---- max-pooling at listed pooled positions -----------------------------------------------
// next_flags != nullptr: the pooled map feeds a convolution layer whose stored previous input is
// this very map; compare each recomputed value with the one it replaces against next_tau and set
// the position's byte in that layer's change map (one byte per pixel, zero on entry).
// next_force != 0: flag every recomputed position (first frame).
hipError_t pool_sparse(hipStream_t st, const int *list, const int *count, int max_count, const float *in,
                       float *pooled, int Ms, int k, int Wo, int No, int Wp, int Np, unsigned char *next_flags,
                       float next_tau, int next_force);

// ---- stored map -> caller's planar output --------------------------------------------------
hipError_t map_to_planar(hipStream_t st, const float *map, float *planar, int M, int Ms, int No, int S);

// helpers
hipError_t fill_iota(hipStream_t st, int *list, int n);

} // namespace cbk
