// Gathered matrix generation + matrix multiplication + output update for gfx950.
//
// Section 3.1 of the paper assembles only the columns of the image matrix X that belong to
// output positions needing an update, multiplies them with the unchanged filter matrix K and
// writes the result (with the activation) over the stored output.  Here the three steps are one
// kernel: a workgroup owns BN output positions to recompute x BM output channels, builds the
// BN x 128-byte slices of the reduced X directly in LDS by gathering 16-byte channel units from
// the channel-contiguous input map, multiplies on the matrix cores and scatters bias + ReLU
// results straight into the stored map.  The reduced X never exists in HBM.
//
// Which positions: from an index list, or -- for maps small enough to be held in LDS -- from the
// map itself.  Every workgroup then loads the map of positions to recompute (or the layer's
// change map, which it first dilates by the filter support), ranks it with popcounts and a scan,
// and picks the positions whose rank falls into its tile: the index extraction and the dilation
// of Section 3.1 without launches of their own.
//
// The workgroup has twelve waves with two roles.  The last four ("producers") compute gather
// addresses, load the next K slices of both operands from global memory and store them to LDS;
// the first eight ("consumers") only read LDS fragments and issue MFMAs (v_mfma_f32_16x16x4_f32
// for float32 storage, v_mfma_f32_16x16x32_bf16 for bfloat16; float32 accumulation either way).
// One producer and two consumer waves share each SIMD, so address arithmetic, global-load latency
// and LDS stores overlap the matrix pipeline instead of draining it once per slice, and while one
// consumer wave waits for its fragments the other keeps the pipeline fed (measured +2.5 % over
// one consumer wave per SIMD).
//
// Work distribution: one workgroup per compute unit.  Output tiles are dealt out whole as long
// as every workgroup gets one; the (tiles mod workgroups) left over are cut along K into
// equal iteration ranges, one per workgroup, so that all compute units finish together whatever
// the number of positions is.  A workgroup that computed only part of a tile's K range stores its
// partial accumulators; the last workgroup to finish a tile (an atomic ticket, nobody waits)
// adds all parts in ascending K order, which keeps results deterministic, and performs the
// output update.
//
// Layers with short filter-matrix rows and few output channels (a first layer on camera frames, 1x1
// layers) would spend such a launch filling and draining the ring; they run gemm_thin_kernel, in
// which every wave multiplies 16 positions by the whole reduction out of its own registers.
#include "kernels.h"

#include <cstdio>
#include <cstdlib>

namespace cbk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef floatx4 floatx4_a4 __attribute__((aligned(4))); // a 16-byte unit that starts at any 4-byte word
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Partial accumulators cross between workgroups that may sit on different XCDs (separate L2s).
// They are written and read with buffer instructions carrying the sc1 bit: write-through to, and
// read at, the level all XCDs share, so no cache-wide write-back or invalidate is needed.
static constexpr int kDeviceCoherent = 0x10; // cache-policy operand: sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slab_resource(const float *p, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p), 0, bytes, 0x00020000);
}


static constexpr int BK = 32;       // K slice per pipeline stage: 128 bytes = 32 floats or 64 bfloat16,
                                    // i.e. 8 units of 16 bytes
static constexpr int KU = 8;        // units per slice
static constexpr int LDK = BK;      // LDS row pitch in 4-byte words: 128 bytes, no padding.  The eight 16-byte
                                    // units of a row are stored permuted (unit u of row r sits in slot
                                    // u ^ lds_swizzle(r)) so that the 16-lane groups of a ds_read_b128
                                    // (16 rows, one or two neighbouring units) and of a ds_write_b128 (two rows,
                                    // all units) each cover all 64 banks once
static constexpr int kConsWaves = 8;              // consumer waves per workgroup (two per SIMD)
static constexpr int NPROD = 64 * 4;              // producer threads (one wave per SIMD)
static constexpr int kRP = NPROD / 8;             // tile rows staged per pass: eight threads (units) per row
static constexpr int NCONS = 64 * kConsWaves;     // consumer threads: waves 0 .. kConsWaves-1
static constexpr int NT = NCONS + NPROD;          // threads per workgroup
static constexpr int kStagedRing = 3; // K slices resident in LDS when the producers stage them through registers
static constexpr int kThreeSetsUnits = 6; // (register staging) tiles whose producer threads load at most this many 16-byte
                                          // units per slice keep three register sets of loads in flight, the others two
static constexpr int kEpiChunk = 4;       // accumulators whose replaced values are loaded together in the output update
static constexpr int kMinIters = 8;       // shortest K range worth giving to a workgroup
static constexpr int kMaxGrid = 1024;
static constexpr int kSmallTileFactor = 2; // big tiles are used from (workgroups / this) big tiles on

static constexpr int kSelMaxWords = 2048; // largest selection map ranked in-kernel (131072 pixels)
static constexpr int kSelWordsPerThread = (kSelMaxWords + NT - 1) / NT;
static constexpr int kSelSlots = kSelWordsPerThread * NT; // LDS words per ranking array (>= kSelMaxWords)

// LDS of one tile shape: a ring of STAGES K slices of both operands, then the tile's pixel list,
// the ticket and two ints for the tile selection.
template <int BM, int BN, int STAGES>
struct TileSmem {
    static constexpr int a_floats = BN * LDK;
    static constexpr int b_floats = BM * LDK;
    static constexpr int tile_bytes = STAGES * (a_floats + b_floats) * 4 + BN * 4 + 16;
};
// LDS of a kernel instantiation (a big and a small tile shape share it): behind the larger of the
// two tiles the selection map's words, their exclusive ranks, and the wave totals of the scan.
template <int BM, int BNB, int SB, int BNS, int SS>
struct KernelSmem {
    static constexpr int tb = TileSmem<BM, BNB, SB>::tile_bytes, ts = TileSmem<BM, BNS, SS>::tile_bytes;
    static constexpr int sel_offset = ((tb > ts ? tb : ts) + 15) / 16 * 16;
    static constexpr int bytes = sel_offset + kSelSlots * 12 + 64;
    static_assert(bytes <= 160 * 1024, "a workgroup has 160 KiB of LDS");
};

// Selection-map mode: the words of the map and the rank of each word's first set bit, in LDS.
struct Selection {
    const uint64_t *words; // nullptr: list mode
    const int *rank;
    int nwords;
};

// A map of nw words (64 positions each) from global memory into LDS as a bitmap.  bytes != 0: the
// map has one byte per position and is packed on the way -- for eight of them in a 64-bit value x
// the high bits of (x | (x & 0x7f..7f) + 0x7f..7f) mark the nonzero bytes and the multiplication
// gathers the eight marks into one byte, which is byte i of the bitmap.  The caller synchronises.
__device__ __forceinline__ void load_bitmap(const uint64_t *__restrict__ map, int bytes, int nw, uint64_t *sM)
{
    const int tid = threadIdx.x;
    if (bytes) {
        unsigned char *sB = reinterpret_cast<unsigned char *>(sM);
        const int n8 = nw * 8;
        for (int i0 = 0; i0 < n8; i0 += 4 * NT) {
            uint64_t x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * NT + tid;
                x[j] = i < n8 ? map[i] : 0ull;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * NT + tid;
                const uint64_t nz =
                    ((x[j] | ((x[j] & 0x7f7f7f7f7f7f7f7full) + 0x7f7f7f7f7f7f7f7full)) & 0x8080808080808080ull) >> 7;
                if (i < n8) sB[i] = (unsigned char)((nz * 0x0102040810204080ull) >> 56);
            }
        }
    } else {
        for (int i0 = 0; i0 < nw; i0 += 4 * NT) {
            uint64_t x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * NT + tid;
                x[j] = i < nw ? map[i] : 0ull;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * NT + tid;
                if (i < nw) sM[i] = x[j];
            }
        }
    }
}

// Bits [a, a + len) of an LDS bitmap as the low bits of the result; 1 <= len <= 64, a >= 0.  Reads
// the word holding bit a and the one behind it, so a zero word must follow the map; no branches.
__device__ __forceinline__ uint64_t lds_bit_run(const uint64_t *m, int a, int len)
{
    const int w = a >> 6, o = a & 63;
    const uint64_t lo = m[w], hi = m[w + 1];
    const uint64_t v = (lo >> o) | ((hi << 1) << (63 - o));
    return v & (~0ull >> (64 - len));
}

// Dilation by the filter support for a stride-1 layer (Section 3.1, second formula), in two
// separable steps on bitmaps in LDS.  sC: change bitmap over the input positions
// [(st*H + iy)*W + ix].  Step 1 writes sH over [(st*H + iy)*Wo + qx]: is any changed pixel in row
// iy under the kw taps of output column qx.  Step 2 (dilated_word_rows) ORs the kh rows of sH that an
// output row reads.  All bitmaps are followed by a zero word.
__device__ __forceinline__ uint64_t row_dilated_word(const GemmArgs &a, const uint64_t *sC, int v, int total)
{
    const int p0 = v * 64, p1 = p0 + 64 < total ? p0 + 64 : total;
    uint64_t res = 0;
    int pos = p0;
    int row = fast_div(pos, a.dWo), x = pos - row * a.Wo; // row = st*H + iy
    while (pos < p1) {
        const int len = a.Wo - x < p1 - pos ? a.Wo - x : p1 - pos;
        // window of input columns xs .. xs + L - 1 of that row; output column x + t reads t .. t + kw - 1
        const int xs = x - a.pad, L = len + a.kw - 1;
        const int k0 = xs < 0 ? -xs : 0, k1 = L < a.W - xs ? L : a.W - xs;
        uint64_t lo = 0, hi = 0;
        if (k1 > k0) {
            const int base = row * a.W + xs;
            if (k0 < 64) lo = lds_bit_run(sC, base + k0, (k1 < 64 ? k1 : 64) - k0) << k0;
            if (k1 > 64) {
                const int s0 = k0 > 64 ? k0 : 64;
                hi = lds_bit_run(sC, base + s0, k1 - s0) << (s0 - 64);
            }
        }
        // OR of the kw shifted copies of the (up to 79-bit) window, by doubling
        int cover = 1;
        while (cover * 2 <= a.kw) {
            lo |= (lo >> cover) | (hi << (64 - cover));
            hi |= hi >> cover;
            cover *= 2;
        }
        if (cover < a.kw) {
            const int sft = a.kw - cover;
            lo |= (lo >> sft) | (hi << (64 - sft));
        }
        if (len < 64) lo &= (1ull << len) - 1ull;
        res |= lo << (pos - p0);
        pos += len;
        x = 0; // a segment ends at the end of its row or of the word
        ++row;
    }
    return res;
}

// The share of tap rows j0, j0 + dj, j0 + 2 dj, ... in word w of the update map: for each output row
// the word touches, the bits of the sH rows qy - pad + j (nothing for rows outside the image).
__device__ __forceinline__ uint64_t dilated_word_rows(const GemmArgs &a, const uint64_t *sH, int w, int j0, int dj,
                                                      int total)
{
    const int p0 = w * 64, p1 = p0 + 64 < total ? p0 + 64 : total;
    const int Ho = a.dHo.d;
    uint64_t res = 0;
    int pos = p0;
    const int orow = fast_div(pos, a.dWo);
    int x = pos - orow * a.Wo, st = fast_div(orow, a.dHo), qy = orow - st * Ho;
    while (pos < p1) {
        const int len = a.Wo - x < p1 - pos ? a.Wo - x : p1 - pos;
        uint64_t r = 0;
        for (int j = j0; j < a.kh; j += dj) {
            const int iy = qy - a.pad + j;
            const bool in = (unsigned)iy < (unsigned)a.H;
            const uint64_t b = lds_bit_run(sH, in ? (st * a.H + iy) * a.Wo + x : 0, len);
            r |= in ? b : 0ull;
        }
        res |= r << (pos - p0);
        pos += len;
        x = 0;
        if (++qy == Ho) {
            qy = 0;
            ++st;
        }
    }
    return res;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves: shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of a row into the next row (rows 1 and 3)
// and lane 31 into rows 2 and 3.  Lanes without a source add the zero given as the old value.
__device__ __forceinline__ int wave_inclusive_sum(int x)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false); // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false); // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false); // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false); // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false); // row_bcast:15
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false); // row_bcast:31
    return x;
}

// Brings the map of positions to recompute into LDS (sW) and ranks it: sRank[i] = number of
// selected positions in the words before word i.  Returns the number of selected positions.
// The map is either given (bits or bytes) or, sel_dilate != 0, derived here from the layer's
// change map by dilation (scratch: LDS that the tile ring will use later); workgroup 0 then also
// writes it to a.upd_out for the kernels that follow.  All NT threads take part; thread t ranks
// the kSelWordsPerThread consecutive words starting at kSelWordsPerThread * t.
__device__ __forceinline__ int rank_selection(const GemmArgs &a, uint64_t *sW, int *sRank, int *sTot,
                                              uint64_t *scratch)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = a.sel_words;
    uint64_t w[kSelWordsPerThread];
    if (a.sel_dilate) {
        const int in_words = a.sel_in_words;
        const int hd_total = a.S * a.H * a.Wo, hd_words = (hd_total + 63) >> 6;
        uint64_t *sC = scratch, *sH = scratch + in_words + 2;
        load_bitmap(a.sel_map, a.sel_bytes, in_words, sC);
        if (tid < 2) sC[in_words + tid] = 0ull;
        __syncthreads();
        for (int v = tid; v < hd_words; v += NT) sH[v] = row_dilated_word(a, sC, v, hd_total);
        if (tid < 2) sH[hd_words + tid] = 0ull;
        for (int i = tid; i < nw; i += NT) sW[i] = 0ull;
        __syncthreads();
        // 2^sh threads per word share its kh tap rows (as many as keeps all words in one round, at
        // most one thread per row); their parts are OR-ed together in LDS
        const int out_total = a.S * a.No;
        int sh = 0;
        while ((1 << sh) < a.kh && (nw << (sh + 1)) <= NT) ++sh;
        for (int t = tid; t < (nw << sh); t += NT) {
            const int i = t >> sh, j0 = t & ((1 << sh) - 1);
            const uint64_t d = dilated_word_rows(a, sH, i, j0, 1 << sh, out_total);
            if (d) atomicOr(reinterpret_cast<unsigned long long *>(sW + i), (unsigned long long)d);
        }
        if (blockIdx.x == 0) {
            __syncthreads();
            for (int i = tid; i < nw; i += NT) a.upd_out[i] = sW[i];
        }
    } else {
        load_bitmap(a.sel_map, a.sel_bytes, nw, sW);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSelWordsPerThread; ++j) {
        const int i = kSelWordsPerThread * tid + j;
        w[j] = i < nw ? sW[i] : 0ull;
    }
    __syncthreads(); // every thread has read its words before they are rewritten below
#pragma unroll
    for (int j = 0; j < kSelWordsPerThread; ++j) sW[kSelWordsPerThread * tid + j] = w[j]; // zero beyond the map
    int c[kSelWordsPerThread], sum = 0;
#pragma unroll
    for (int j = 0; j < kSelWordsPerThread; ++j) {
        c[j] = __popcll(w[j]);
        sum += c[j];
    }
    const int incl = wave_inclusive_sum(sum);
    if (lane == 63) sTot[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        const int t = sTot[i];
        if (i < wave) before += t;
        total += t;
    }
    int e = before + incl - sum;
#pragma unroll
    for (int j = 0; j < kSelWordsPerThread; ++j) {
        sRank[kSelWordsPerThread * tid + j] = e;
        e += c[j];
    }
    __syncthreads();
    return total;
}

// The selected pixels of rank r0 .. r0 + BN - 1 into sU (-1 where the selection ends before).
// sRange: two ints of LDS.  All NT threads take part.
template <int BN>
__device__ __forceinline__ void select_tile(const Selection &sel, int n, int r0, int *sU, int *sRange)
{
    const int tid = threadIdx.x;
    const int r1 = (r0 + BN < n ? r0 + BN : n) - 1; // last rank wanted (r0 <= r1: the tile is not empty)
    for (int i = tid; i < BN; i += NT) sU[i] = -1;
    // the words holding rank r0 and rank r1: each is found by the one thread that ranks it
#pragma unroll
    for (int j = 0; j < kSelWordsPerThread; ++j) {
        const int i = kSelWordsPerThread * tid + j;
        const int e = sel.rank[i], c = __popcll(sel.words[i]);
        if (e <= r0 && r0 < e + c) sRange[0] = i;
        if (e <= r1 && r1 < e + c) sRange[1] = i;
    }
    __syncthreads();
    const int wlo = sRange[0], whi = sRange[1];
    // one lane per pixel of those words
    for (int idx = tid; idx < (whi - wlo + 1) * 64; idx += NT) {
        const int i = wlo + (idx >> 6), b = idx & 63;
        const uint64_t bits = sel.words[i];
        if ((bits >> b) & 1ull) {
            const int r = sel.rank[i] + __popcll(bits & ((1ull << b) - 1ull)) - r0;
            if ((unsigned)r < (unsigned)BN) sU[r] = i * 64 + b;
        }
    }
}

// The split of one launch's work over W workgroups; a pure function of its arguments.  32-bit
// arithmetic: W <= 1024 and the host refuses filter matrices of 2^20 slices or more, so
// rem * nk stays below 2^30.
struct Schedule {
    int tiles; // output tiles: pixel tiles x channel tiles (channel tile fastest)
    int whole; // rounds in which every workgroup takes one whole tile
    int rem;   // tiles left over, shared along K
    int wr;    // workgroups sharing the left-over tiles
    int iters; // rem * nk: K-slice iterations of the left-over tiles
    int q, r;  // iters = q * wr + r
};

__device__ __forceinline__ Schedule make_schedule(int n, int bn, int mtiles, int nk, const FastDiv &dW)
{
    const int W = dW.d;
    Schedule s;
    s.tiles = ((n + bn - 1) / bn) * mtiles;
    s.whole = fast_div(s.tiles, dW);
    s.rem = s.tiles - s.whole * W;
    s.iters = s.rem * nk;
    // Cut every left-over tile into the same number of parts if that occupies at least 7/8 of
    // the workgroups (ranges then start on tile boundaries: one segment per workgroup); otherwise
    // deal the iterations out evenly over all workgroups.  Never make parts shorter than
    // kMinIters slices.
    const int max_parts = nk / kMinIters > 1 ? nk / kMinIters : 1;
    int wr = 1;
    if (s.rem > 0) {
        int p = W / s.rem;
        if (p > max_parts) p = max_parts;
        if (p < 1) p = 1;
        wr = s.rem * p;
        if (wr * 8 < W * 7 && s.rem * max_parts >= W) wr = W;
        if (wr > W) wr = W;
    }
    s.wr = wr;
    s.q = s.iters / wr;
    s.r = s.iters - s.q * wr;
    return s;
}

// First iteration of workgroup w's share: floor(iters * w / wr), and the workgroup owning an iteration.
__device__ __forceinline__ int share_begin(const Schedule &s, int w) { return s.q * w + s.r * w / s.wr; }

__device__ __forceinline__ int share_owner(const Schedule &s, int it)
{
    // estimate in float (off by one at most for these magnitudes), then settle exactly
    int w = (int)((float)it * (float)s.wr / (float)s.iters);
    if (w > s.wr - 1) w = s.wr - 1;
    if (w < 0) w = 0;
    while (w + 1 < s.wr && share_begin(s, w + 1) <= it) ++w;
    while (w > 0 && share_begin(s, w) > it) --w;
    return w;
}

// Image-matrix rows gathered by one producer thread for one K slice: PA rows (32 apart), one
// 16-byte unit each.  tp is the slice's tap descriptor for this thread's unit column.
template <int PA>
__device__ __forceinline__ void gather_rows(const GemmArgs &a, const int2 tp, const int (&iy0)[PA],
                                            const int (&ix0)[PA], const int (&base)[PA], floatx4 (&ra)[PA])
{
    const float *x = static_cast<const float *>(a.x); // 4-byte words, whatever the storage type
    const int tj = tp.y & 0xff, ti = (tp.y >> 8) & 0xff;
    const bool tv = (tp.y >> 16) != 0;
#pragma unroll
    for (int ps = 0; ps < PA; ++ps) {
        const bool ok = tv && (unsigned)(iy0[ps] + tj) < (unsigned)a.H && (unsigned)(ix0[ps] + ti) < (unsigned)a.W;
        // outside the image (or no pixel in this row): the zero unit kept behind the map, so that the
        // load needs no predication and the registers no clearing
        const unsigned idx = ok ? (unsigned)(base[ps] + tp.x) : (unsigned)a.zero_word;
        ra[ps] = *reinterpret_cast<const floatx4_a4 *>(x + idx);
    }
}

// wrow: this thread's unit column in its first filter-matrix row; krow = units per row.
template <int BM, int PB>
__device__ __forceinline__ void load_filter_rows(const floatx4 *wrow, int krow, int kc, int r0, floatx4 (&rb)[PB])
{
    if constexpr (BM >= kRP) {
#pragma unroll
        for (int ps = 0; ps < PB; ++ps) rb[ps] = wrow[(size_t)(kRP * ps) * krow + kc * KU];
    } else {
        if (r0 < BM) rb[0] = wrow[kc * KU];
    }
}

__device__ __forceinline__ int lds_swizzle(int row) { return (row >> 1) & 7; }

// v: this thread's slot in the row, i.e. its unit column already permuted for row r0 (rows 32 apart
// share the permutation).
template <int BM, int PA, int PB>
__device__ __forceinline__ void stage_rows(float *A, float *B, int r0, int v, const floatx4 (&ra)[PA],
                                           const floatx4 (&rb)[PB])
{
#pragma unroll
    for (int ps = 0; ps < PA; ++ps) *reinterpret_cast<floatx4 *>(A + (r0 + kRP * ps) * LDK + v * 4) = ra[ps];
    if constexpr (BM >= kRP) {
#pragma unroll
        for (int ps = 0; ps < PB; ++ps) *reinterpret_cast<floatx4 *>(B + (r0 + kRP * ps) * LDK + v * 4) = rb[ps];
    } else {
        if (r0 < BM) *reinterpret_cast<floatx4 *>(B + r0 * LDK + v * 4) = rb[0];
    }
}

// s_waitcnt vmcnt(N), everything else unconstrained (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a six-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// The workgroup barrier as the direct-to-LDS producers execute it: the bare instruction.  The
// fences of __syncthreads() would make the wave wait for all of its loads in flight, which are
// exactly what has to stay in flight across the barrier; the one ordering the producers owe the
// consumers -- a slice has landed in LDS before the barrier that publishes it -- is the explicit
// wait_vmcnt in front of it, and the compiler must not move memory operations across either.
__device__ __forceinline__ void producer_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

typedef __attribute__((address_space(1))) const void *GlobalPtr;
typedef __attribute__((address_space(3))) void *LdsPtr;

// Producer waves, direct-to-LDS variant: global_load_lds_dwordx4 moves 16 bytes per lane from
// global memory into LDS without passing through registers -- lane l of an instruction lands at
// the wave-uniform LDS base + 16 l, i.e. in slot l & 7 of row l >> 3 of eight consecutive rows --
// so the producers only compute addresses.  Wave pw covers rows 8 pw .. 8 pw + 7 of every pass of
// kRP rows; vf is the unit column this lane fetches (its slot with the row permutation undone).
// The ring holds STAGES slices: slice kc + STAGES - 1 is issued in iteration kc into the slot
// that slice kc - 1 occupied, and has to have landed by the barrier that ends iteration
// kc + STAGES - 3 (the consumers read the first fragments of a slice one iteration early).  The
// loads of a wave complete in order, so "at most (STAGES - 3) slices' worth of instructions
// outstanding" means slice kc + 2 is in LDS.  No LDS reads and no other vector memory
// instructions occur in this loop, which keeps the instruction count per slice exact.
// While two consumer waves keep the matrix pipeline of a SIMD busy, a vector-ALU instruction of the
// producer wave on that SIMD gets issued about once per MFMA (measured: 40 cycles per instruction),
// so the producers' instruction count per slice, not the memory system, is what can hold up the loop.
// Hence: everything wave-uniform is computed on the scalar unit (the ring slot and the LDS
// destinations; with UT also the filter tap of the slice), filter rows are addressed as a uniform
// base plus a per-lane 32-bit offset that never changes, and what is left per image-matrix row is
// the bounds test of its tap and the choice between the pixel's address and the zero unit.
// UT ("uniform tap"): the units per pixel are a multiple of the eight units of a slice, so a slice
// lies inside one filter tap and the tap is the same for all lanes; base[] then already contains
// the lane's own unit offset.
template <int DT, int BM, int BN, int STAGES, int PA, bool UT>
__device__ __forceinline__ void direct_producer(const GemmArgs &a, float *As, float *Bs, int kc0, int kc1, int mt,
                                                int krow, int pw_, int r0, int vf, const int (&iy0)[PA],
                                                const int (&ix0)[PA], const int (&base)[PA])
{
    constexpr int PB = (BM + kRP - 1) / kRP; // filter-row passes (a tile of 16 channels: two waves repeat the others' rows)
    constexpr int PS = PA + PB;              // instructions per slice and wave
    constexpr int ASZ = BN * LDK, BSZ = BM * LDK;
    static_assert((STAGES - 3) * PS < 64, "outstanding loads must fit the counter");
    const int pw = __builtin_amdgcn_readfirstlane(pw_); // the wave's number among the producers, as a scalar
    const float *x = static_cast<const float *>(a.x);
    // this channel tile's rows of the filter matrix; the lane's rows and unit as byte offsets from there
    // (below 4 GiB: the host checks BM * Kpad)
    const char *wtile = reinterpret_cast<const char *>(static_cast<const floatx4 *>(a.wt) + (size_t)mt * BM * krow);
    unsigned wofs[PB];
#pragma unroll
    for (int ps = 0; ps < PB; ++ps) wofs[ps] = (unsigned)((r0 % BM + kRP * ps) * krow + vf) * 16u;
    auto issue = [&](int kc, int slot) {
        // tap of this lane's unit in slice kc: unit index -> (filter tap, channel unit) -> (j, i)
        const int q = kc * KU + (UT ? 0 : vf);
        const int tap = fast_div(q, a.dVin), cu = q - tap * a.dVin.d;
        const int tj = fast_div(tap, a.dKw), ti = tap - tj * a.kw;
        const bool tv = tj < a.kh;
        const int off = (tj * a.W + ti) * a.pix_words + cu * 4;
        float *A = As + slot * ASZ + pw * 8 * LDK, *B = Bs + slot * BSZ + (pw * 8 % BM) * LDK;
#pragma unroll
        for (int ps = 0; ps < PA; ++ps) {
            const bool ok = tv && (unsigned)(iy0[ps] + tj) < (unsigned)a.H && (unsigned)(ix0[ps] + ti) < (unsigned)a.W;
            // outside the image (or no pixel in this row): the zero unit kept behind the map, so that the
            // load needs no predication
            const unsigned idx = ok ? (unsigned)(base[ps] + off) : (unsigned)a.zero_word;
            __builtin_amdgcn_global_load_lds((GlobalPtr)(x + idx), (LdsPtr)(A + kRP * ps * LDK), 16, 0, 0);
        }
        const char *wslice = wtile + (size_t)kc * (KU * 16);
#pragma unroll
        for (int ps = 0; ps < PB; ++ps)
            __builtin_amdgcn_global_load_lds((GlobalPtr)(wslice + wofs[ps]), (LdsPtr)(B + kRP * ps * LDK), 16, 0, 0);
    };
    // Nothing of this wave is in flight here; saying so keeps the compiler, which tracks loads into
    // registers along every path through the kernel, from waiting for imagined ones inside the loop.
    wait_vmcnt<0>();
    // prologue: STAGES - 1 slices in flight, the first two landed
#pragma unroll
    for (int d = 0; d < STAGES - 1; ++d)
        if (kc0 + d < kc1) issue(kc0 + d, d);
    if (kc0 + STAGES - 2 < kc1)
        wait_vmcnt<(STAGES - 3) * PS>();
    else
        wait_vmcnt<0>();
    producer_barrier();
    int slot = STAGES - 1; // ring slot of slice kc + STAGES - 1
    for (int kc = kc0; kc < kc1; ++kc) {
        if (kc + STAGES - 1 < kc1) {
            issue(kc + STAGES - 1, slot);
            wait_vmcnt<(STAGES - 3) * PS>();
        } else {
            wait_vmcnt<0>();
        }
        slot = slot == STAGES - 1 ? 0 : slot + 1;
        producer_barrier();
    }
}

// BM x BN workgroup tile; the consumer waves are arranged WM (channels) x WN (pixels).
//
// LDS holds a ring of three K slices.  In iteration kc the producers store slice kc+2 and issue
// the global loads of a slice two or three further on (one per register set), while the consumers
// multiply slice kc and already read the first fragments of slice kc+1, so the matrix pipeline
// keeps running across the one barrier per slice.
template <int DT, int BM, int BN, int WM, int WN, int STAGES, bool DIRECT>
__device__ __forceinline__ void gemm_gather_body(const GemmArgs &a, const int n, float *smem, const Selection sel)
{
    static_assert(WM * WN == kConsWaves, "one sub-tile per consumer wave");
    static_assert(DIRECT ? STAGES >= 3 : STAGES == kStagedRing, "ring depth");
    constexpr int TP = BN / WN / 16; // 16-pixel MFMA tiles per consumer wave
    constexpr int TC = BM / WM / 16; // 16-channel MFMA tiles per consumer wave
    constexpr int PA = BN / kRP;     // image-matrix rows staged per producer thread and slice
    constexpr int PB = (BM + kRP - 1) / kRP;
    constexpr int NS = PA + PB <= kThreeSetsUnits ? 3 : 2; // (register staging) sets of loads in flight per producer thread
    static_assert(BN % kRP == 0, "whole passes over the pixel rows");
    constexpr int ASZ = BN * LDK, BSZ = BM * LDK;
    constexpr int SLAB = BM * BN; // floats of one partial-accumulator slab
    static_assert(TP >= 1 && TC >= 1, "tile too small");
    static_assert(BK == 32, "two 16-wide fragment groups per slice");
    static_assert(TC * TP * 4 * NCONS == SLAB, "a slab holds every consumer lane's accumulators");

    float *As = smem;                                     // [STAGES][BN][LDK]  gathered image-matrix slices
    float *Bs = smem + STAGES * ASZ;                      // [STAGES][BM][LDK]  filter-matrix slices
    int *sU = reinterpret_cast<int *>(Bs + STAGES * BSZ); // [BN] listed pixels of this tile (-1: none)
    int *sFlag = sU + BN;                                  // ticket of the tile just finished

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const bool producer = wave >= kConsWaves;

    const int mtiles = a.Mpad / BM;
    const int krow = a.Kpad / Unit<DT>::N; // units per filter-matrix row
    const int nk = krow / KU;
    const int W = gridDim.x;
    const Schedule sch = make_schedule(n, BN, mtiles, nk, a.dGrid);
    if (sch.tiles == 0) return;
    // Workgroups are dealt round-robin over the 8 XCDs.  Number them so that each XCD works on a
    // contiguous range of tiles / iterations: neighbours share gathered pixels (channel tiles of
    // one pixel tile) or filter slices, and that sharing then happens inside one L2.
    const int w = (int)(blockIdx.x & 7) * (W >> 3) + (int)(blockIdx.x >> 3);
    const bool xcd_ranges = (sch.wr & 7) == 0;
    const int wsh = xcd_ranges ? (int)(blockIdx.x & 7) * (sch.wr >> 3) + (int)(blockIdx.x >> 3)
                               : (int)blockIdx.x; // number inside the K-sharing group
    const bool sharing =
        sch.rem > 0 && (xcd_ranges ? (int)(blockIdx.x >> 3) < (sch.wr >> 3) : (int)blockIdx.x < sch.wr);
    const int it_begin = sharing ? share_begin(sch, wsh) : 0;
    const int it_end = sharing ? share_begin(sch, wsh + 1) : 0;

    int round = 0;
    int it = it_begin;
    while (true) {
        // ---- next segment of this workgroup: a whole tile, or part of a shared tile's K range
        int tile, kc0, kc1, shared_j = -1;
        if (round < sch.whole) {
            tile = round * W + w;
            kc0 = 0;
            kc1 = nk;
            ++round;
        } else if (it < it_end) {
            shared_j = fast_div(it, a.dNk);
            kc0 = it - shared_j * nk;
            const int left = it_end - it;
            kc1 = (left < nk - kc0) ? kc0 + left : nk;
            tile = sch.whole * W + shared_j;
            it += kc1 - kc0;
        } else {
            break;
        }
        const int pt = tile / mtiles;
        const int mt = tile - pt * mtiles;
        const bool partial = (kc1 - kc0) != nk;

        // Producers: the tap descriptors of the first slices do not depend on the tile's pixel list,
        // so their loads are in flight while the list is made.
        const int ptid = producer ? tid - NCONS : 0;
        const int v = ptid & 7;   // 16-byte unit column inside the K slice
        const int r0 = ptid >> 3; // first row this thread stages
        const floatx4 *wrow = static_cast<const floatx4 *>(a.wt) + (size_t)(mt * BM + r0) * krow + v;
        const int2 *taps = a.taps + v;
        auto tap = [&](int kc) { return taps[(kc < kc1 ? kc : kc0) * KU]; };
        int2 tp0, tp1, tp[NS];
        if (producer && !DIRECT) {
            tp0 = tap(kc0);
            tp1 = tap(kc0 + 1);
#pragma unroll
            for (int u = 0; u < NS; ++u) tp[u] = tap(kc0 + 2 + u);
        }
        __syncthreads(); // the previous segment's LDS reads are done
        if (sel.words) {
            select_tile<BN>(sel, n, pt * BN, sU, sFlag + 1);
        } else {
            for (int i = tid; i < BN; i += NT) {
                const int u = pt * BN + i;
                sU[i] = (u < n) ? a.list[u] : -1;
            }
        }
        __syncthreads();

        // consumer coordinates (used again after the role-specific loops)
        const int cw = producer ? 0 : wave;
        const int wpx0 = (cw % WN) * (BN / WN);
        const int wch0 = (cw / WN) * (BM / WM);
        const int lrow = lane & 15; // row of the 16-row operand tiles this lane feeds
        const int lk = lane >> 4;   // k slot this lane feeds
        // cleared inside the role branches, for the producers after their loop: registers that
        // hold nothing while they stage slices
        floatx4 acc[TC][TP];

        // Both roles execute the same number of barriers: one after the prologue, one per slice.
        if (producer) {
            // staging through registers: this thread loads unit column v and stores it to slot vs;
            // direct to LDS: the hardware puts lane l's 16 bytes into slot l & 7 of row l >> 3 of the
            // eight rows an instruction covers, so the thread fetches the unit that belongs there
            const int vs = v ^ lds_swizzle(r0);
            int iy0[PA], ix0[PA], base[PA];
#pragma unroll
            for (int ps = 0; ps < PA; ++ps) {
                const int g = sU[r0 + kRP * ps];
                if (g >= 0) {
                    const int st = fast_div(g, a.dNo), q = g - st * a.No;
                    const int qy = fast_div(q, a.dWo), qx = q - qy * a.Wo;
                    iy0[ps] = qy * a.stride - a.pad;
                    ix0[ps] = qx * a.stride - a.pad;
                    base[ps] = ((st * a.H + iy0[ps]) * a.W + ix0[ps]) * a.pix_words;
                } else {
                    iy0[ps] = -(1 << 28);
                    ix0[ps] = -(1 << 28);
                    base[ps] = 0;
                }
            }
            if constexpr (DIRECT) {
                if ((a.dVin.d & (KU - 1)) == 0) {
                    // a slice lies inside one filter tap: the lane's unit goes into its pixel offsets once
#pragma unroll
                    for (int ps = 0; ps < PA; ++ps) base[ps] += vs * 4;
                    direct_producer<DT, BM, BN, STAGES, PA, true>(a, As, Bs, kc0, kc1, mt, krow, wave - kConsWaves, r0, vs, iy0,
                                                                  ix0, base);
                } else {
                    direct_producer<DT, BM, BN, STAGES, PA, false>(a, As, Bs, kc0, kc1, mt, krow, wave - kConsWaves, r0, vs,
                                                                   iy0, ix0, base);
                }
            } else {
            // NS register sets: in iteration kc the slice kc+2, loaded NS iterations ago, is stored to
            // the LDS ring and the loads of slice kc+2+NS are issued into the same registers.  The
            // loop runs at the pace of these loads when NS slices of MFMA work are shorter than a
            // global-memory round trip, so the small tiles get a third set.  The tap descriptor of
            // a slice is loaded a round before the operand loads that need it.
            floatx4 ra[NS][PA], rb[NS][PB];
            // prologue: slices kc0 and kc0+1 into ring slots 0 and 1, slices kc0+2 .. kc0+1+NS in flight
            gather_rows<PA>(a, tp0, iy0, ix0, base, ra[0]);
            load_filter_rows<BM, PB>(wrow, krow, kc0, r0, rb[0]);
            if (kc0 + 1 < kc1) {
                gather_rows<PA>(a, tp1, iy0, ix0, base, ra[1]);
                load_filter_rows<BM, PB>(wrow, krow, kc0 + 1, r0, rb[1]);
            }
            stage_rows<BM, PA, PB>(As, Bs, r0, vs, ra[0], rb[0]);
            if (kc0 + 1 < kc1) stage_rows<BM, PA, PB>(As + ASZ, Bs + BSZ, r0, vs, ra[1], rb[1]);
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                if (kc0 + 2 + u < kc1) {
                    gather_rows<PA>(a, tp[u], iy0, ix0, base, ra[u]);
                    load_filter_rows<BM, PB>(wrow, krow, kc0 + 2 + u, r0, rb[u]);
                }
                tp[u] = tap(kc0 + 2 + NS + u);
            }
            __syncthreads();
            int slot = 2; // ring slot of slice kc+2
            for (int kc = kc0; kc < kc1; kc += NS) {
#pragma unroll
                for (int u = 0; u < NS; ++u) {
                    if (kc + u < kc1) {
                        if (kc + u + 2 < kc1) {
                            stage_rows<BM, PA, PB>(As + slot * ASZ, Bs + slot * BSZ, r0, vs, ra[u], rb[u]);
                            if (kc + u + 2 + NS < kc1) {
                                gather_rows<PA>(a, tp[u], iy0, ix0, base, ra[u]);
                                load_filter_rows<BM, PB>(wrow, krow, kc + u + 2 + NS, r0, rb[u]);
                                tp[u] = tap(kc + u + 2 + 2 * NS);
                            }
                        }
                        slot = slot == kStagedRing - 1 ? 0 : slot + 1;
                        __syncthreads();
                    }
                }
            }
            } // register staging
#pragma unroll
            for (int j = 0; j < TC; ++j)
#pragma unroll
                for (int i = 0; i < TP; ++i) acc[j][i] = (floatx4){0.f, 0.f, 0.f, 0.f};
        } else {
#pragma unroll
            for (int j = 0; j < TC; ++j)
#pragma unroll
                for (int i = 0; i < TP; ++i) acc[j][i] = (floatx4){0.f, 0.f, 0.f, 0.f};
            // fragment group kk of this lane's row: unit 4*kk + lk, stored in slot (4*kk + lk) ^ swizzle
            const int u0 = (lk ^ lds_swizzle(lrow)) * 4;
            const float *A0 = As + (wpx0 + lrow) * LDK;
            const float *B0 = Bs + (wch0 + lrow) * LDK;
            // Each lane reads four consecutive k of its row; MFMA step s then contracts
            // k = 16*group + 4*slot + s for slot = 0..3 -- both operands use the same permutation.
            // D = (filter rows) x (pixel columns): D[4*slot + r][lane%16] lands in this lane,
            // i.e. four consecutive channels of one pixel per accumulator.
            floatx4 af[2][TP], bf[2][TC];
            auto read_frags = [&](int set, int slot, int kk) {
                const float *A = A0 + slot * ASZ + (u0 ^ (kk * 16));
                const float *B = B0 + slot * BSZ + (u0 ^ (kk * 16));
#pragma unroll
                for (int i = 0; i < TP; ++i) af[set][i] = *reinterpret_cast<const floatx4 *>(A + i * 16 * LDK);
#pragma unroll
                for (int j = 0; j < TC; ++j) bf[set][j] = *reinterpret_cast<const floatx4 *>(B + j * 16 * LDK);
            };
            auto multiply = [&](int set) {
                if constexpr (DT == kBF16) {
                    // one 16-byte fragment = 8 consecutive k: v_mfma_f32_16x16x32_bf16 takes it whole
#pragma unroll
                    for (int j = 0; j < TC; ++j)
#pragma unroll
                        for (int i = 0; i < TP; ++i)
                            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8, bf[set][j]), __builtin_bit_cast(bf16x8, af[set][i]),
                                acc[j][i], 0, 0, 0);
                } else {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int j = 0; j < TC; ++j)
#pragma unroll
                            for (int i = 0; i < TP; ++i)
                                acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[set][j][s], af[set][i][s],
                                                                                 acc[j][i], 0, 0, 0);
                }
            };
            __syncthreads();
            // the wave feeding the matrix pipeline wins instruction-issue arbitration on its SIMD
            __builtin_amdgcn_s_setprio(3);
            read_frags(0, 0, 0);
            int slot = 0; // ring slot of slice kc
            for (int kc = kc0; kc < kc1; ++kc) {
                const int nslot = slot == STAGES - 1 ? 0 : slot + 1;
                // The scheduling barriers pin the order "issue the LDS reads of the next fragment
                // group, then the MFMAs of the current one", so that LDS latency and bandwidth
                // are spent while the matrix pipeline is busy.
                read_frags(1, slot, 1);
                __builtin_amdgcn_sched_barrier(0);
                multiply(0);
                __builtin_amdgcn_sched_barrier(0);
                // Also in the last iteration, where the slot holds nothing of use: under a condition
                // the compiler, which counts outstanding LDS reads per path, would make the MFMAs
                // below wait for these reads too.
                read_frags(0, nslot, 0);
                __builtin_amdgcn_sched_barrier(0);
                multiply(1);
                __builtin_amdgcn_sched_barrier(0);
                slot = nslot;
                __syncthreads();
            }
            __builtin_amdgcn_s_setprio(0);
        }

        // ---- a shared tile: store this K range's accumulators, take a ticket; the workgroup
        //      holding the last ticket adds up all ranges (ascending K) and does the output update.
        //      Slab stores are complete (vmcnt(0)) before the ticket is taken.
        bool finish = true;
        if (partial) {
            const int t0 = shared_j * nk;
            const int w_first = share_owner(sch, t0);
            const int w_last = share_owner(sch, t0 + nk - 1);
            const int ctid = producer ? 0 : tid;
            if (!producer) {
                // slab 2*wsh + (0: first tile this workgroup touches, 1: a later one), register layout:
                // one float4 per lane and accumulator, consecutive lanes consecutive addresses
                const int first_j = fast_div(it_begin, a.dNk);
                const __amdgpu_buffer_rsrc_t slab = slab_resource(
                    a.partial + (size_t)(2 * wsh + (shared_j == first_j ? 0 : 1)) * SLAB, SLAB * 4);
#pragma unroll
                for (int j = 0; j < TC; ++j)
#pragma unroll
                    for (int i = 0; i < TP; ++i)
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, acc[j][i]), slab,
                                                               ((j * TP + i) * NCONS + ctid) * 16, 0, kDeviceCoherent);
                // all of this lane's slab stores have reached the device-coherent level
                __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
            }
            __syncthreads();
            if (tid == 0)
                *sFlag = __hip_atomic_fetch_add(a.tickets + shared_j, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            finish = (*sFlag == w_last - w_first);
            if (finish) {
                if (tid == 0) a.tickets[shared_j] = 0; // ready for the next launch
                if (!producer) {
                    // Sum the parts in ascending K order, whichever workgroup finishes (its own part
                    // is read back like the others, which keeps the accumulators in one register set).
#pragma unroll
                    for (int j = 0; j < TC; ++j)
#pragma unroll
                        for (int i = 0; i < TP; ++i) acc[j][i] = (floatx4){0.f, 0.f, 0.f, 0.f};
                    for (int ww = w_first; ww <= w_last; ++ww) {
                        const int fj = fast_div(share_begin(sch, ww), a.dNk);
                        const __amdgpu_buffer_rsrc_t slab = slab_resource(
                            a.partial + (size_t)(2 * ww + (shared_j == fj ? 0 : 1)) * SLAB, SLAB * 4);
                        floatx4 part[TC][TP];
#pragma unroll
                        for (int j = 0; j < TC; ++j)
#pragma unroll
                            for (int i = 0; i < TP; ++i)
                                part[j][i] = __builtin_bit_cast(
                                    floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                 slab, ((j * TP + i) * NCONS + ctid) * 16, 0, kDeviceCoherent));
#pragma unroll
                        for (int j = 0; j < TC; ++j)
#pragma unroll
                            for (int i = 0; i < TP; ++i) acc[j][i] += part[j][i];
                    }
                }
            }
        }

        // ---- output update: bias, activation, scatter to the stored map; optionally the change
        //      detection of the layer this map feeds (new value against the one it replaces)
        if (finish && !producer) {
            const bool detect = a.next_flags != nullptr && !a.next_force;
            bool changed[TP];
#pragma unroll
            for (int i = 0; i < TP; ++i) changed[i] = false;
            float4 bias[TC];
#pragma unroll
            for (int j = 0; j < TC; ++j) bias[j] = *reinterpret_cast<const float4 *>(a.bias + mt * BM + wch0 + j * 16 + lk * 4);
            // The values about to be replaced are loaded kEpiChunk accumulators at a time before the
            // stores of those accumulators (the compiler cannot move a load across a store to the
            // same map, and one round trip to memory per accumulator would line up at the very end
            // of the kernel).  Accumulator q covers channels of block q / TP at the positions of block q % TP.
            constexpr int CH = TC * TP < kEpiChunk ? TC * TP : kEpiChunk;
            static_assert((TC * TP) % CH == 0, "whole chunks");
#pragma unroll
            for (int q0 = 0; q0 < TC * TP; q0 += CH) {
                uintx4 replaced[CH];
                if (detect) {
#pragma unroll
                    for (int qq = 0; qq < CH; ++qq) {
                        const int j = (q0 + qq) / TP, i = (q0 + qq) % TP;
                        const int ch = mt * BM + wch0 + j * 16 + lk * 4;
                        const int g = sU[wpx0 + i * 16 + lrow];
                        replaced[qq] = (uintx4){0u, 0u, 0u, 0u};
                        if (g >= 0 && ch < a.Ms) {
                            if constexpr (DT == kBF16) {
                                const uint2 v = *reinterpret_cast<const uint2 *>(static_cast<const unsigned short *>(a.out) +
                                                                                 (size_t)g * a.Ms + ch);
                                replaced[qq][0] = v.x;
                                replaced[qq][1] = v.y;
                            } else {
                                replaced[qq] = *reinterpret_cast<const uintx4 *>(static_cast<const float *>(a.out) +
                                                                                 (size_t)g * a.Ms + ch);
                            }
                        }
                    }
                }
#pragma unroll
                for (int qq = 0; qq < CH; ++qq) {
                    const int j = (q0 + qq) / TP, i = (q0 + qq) % TP;
                    const int ch = mt * BM + wch0 + j * 16 + lk * 4;
                    const float4 bv = bias[j];
                    const int g = sU[wpx0 + i * 16 + lrow];
                    if (g >= 0 && ch < a.Ms) {
                        float4 o;
                        o.x = acc[j][i][0] + bv.x;
                        o.y = acc[j][i][1] + bv.y;
                        o.z = acc[j][i][2] + bv.z;
                        o.w = acc[j][i][3] + bv.w;
                        if (a.relu) {
                            o.x = fmaxf(o.x, 0.f);
                            o.y = fmaxf(o.y, 0.f);
                            o.z = fmaxf(o.z, 0.f);
                            o.w = fmaxf(o.w, 0.f);
                        }
                        if constexpr (DT == kBF16) {
                            // four consecutive bfloat16 channels: one 8-byte word
                            uint2 *dst = reinterpret_cast<uint2 *>(static_cast<unsigned short *>(a.out) +
                                                                   (size_t)g * a.Ms + ch);
                            uint2 nv;
                            nv.x = (unsigned)bf16_bits(o.x) | ((unsigned)bf16_bits(o.y) << 16);
                            nv.y = (unsigned)bf16_bits(o.z) | ((unsigned)bf16_bits(o.w) << 16);
                            if (detect) {
                                const uint2 ov = make_uint2(replaced[qq][0], replaced[qq][1]);
                                changed[i] |= fabsf(bf16_value(nv.x & 0xffff) - bf16_value(ov.x & 0xffff)) > a.next_tau ||
                                              fabsf(bf16_value(nv.x >> 16) - bf16_value(ov.x >> 16)) > a.next_tau ||
                                              fabsf(bf16_value(nv.y & 0xffff) - bf16_value(ov.y & 0xffff)) > a.next_tau ||
                                              fabsf(bf16_value(nv.y >> 16) - bf16_value(ov.y >> 16)) > a.next_tau;
                            }
                            *dst = nv;
                        } else {
                            float4 *dst = reinterpret_cast<float4 *>(static_cast<float *>(a.out) + (size_t)g * a.Ms + ch);
                            if (detect) {
                                const float4 ov = make_float4(__uint_as_float(replaced[qq][0]), __uint_as_float(replaced[qq][1]),
                                                              __uint_as_float(replaced[qq][2]), __uint_as_float(replaced[qq][3]));
                                changed[i] |= fabsf(o.x - ov.x) > a.next_tau || fabsf(o.y - ov.y) > a.next_tau ||
                                              fabsf(o.z - ov.z) > a.next_tau || fabsf(o.w - ov.w) > a.next_tau;
                            }
                            *dst = o;
                        }
                    }
                }
            }
            if (a.next_flags) {
#pragma unroll
                for (int i = 0; i < TP; ++i) {
                    const int g = sU[wpx0 + i * 16 + lrow];
                    int f = a.next_force ? 1 : (int)changed[i];
                    // the other channels of this pixel sit in the lanes 16, 32 and 48 further on
                    f |= __shfl_xor(f, 16);
                    f |= __shfl_xor(f, 32);
                    if (lk == 0 && f && g >= 0) a.next_flags[g] = 1;
                }
            }
        }
    }
}

// The kernel: reads the list length (or ranks the selection map) and runs
// the tile shape that suits it -- BNB listed pixels per tile normally, BNS when even the deepest K
// split of the big tiles would leave compute units idle (short lists): small tiles then need no
// or fewer shared tiles, whose partial sums and reduction are pure overhead.
template <int DT, int BM, int BNB, int WMB, int WNB, int SB, bool DB, int BNS, int WMS, int WNS, int SS, bool DS>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu((NT + 255) / 256, (NT + 255) / 256))) void gemm_gather_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) float smem[];
    Selection sel = {nullptr, nullptr, 0};
    int n;
    if (a.sel_words > 0) {
        char *base = reinterpret_cast<char *>(smem) + KernelSmem<BM, BNB, SB, BNS, SS>::sel_offset;
        uint64_t *sW = reinterpret_cast<uint64_t *>(base);
        int *sRank = reinterpret_cast<int *>(base + kSelSlots * 8);
        n = rank_selection(a, sW, sRank, sRank + kSelSlots, reinterpret_cast<uint64_t *>(smem));
        sel.words = sW;
        sel.rank = sRank;
        sel.nwords = a.sel_words;
    } else {
        n = *a.count;
    }
    const long long big_tiles = (long long)((n + BNB - 1) / BNB) * (a.Mpad / BM);
    if (big_tiles * kSmallTileFactor >= (long long)gridDim.x)
        gemm_gather_body<DT, BM, BNB, WMB, WNB, SB, DB>(a, n, smem, sel);
    else
        gemm_gather_body<DT, BM, BNS, WMS, WNS, SS, DS>(a, n, smem, sel);
}

// ---- layers whose whole reduction fits a wave's registers ----------------------------------
//
// A filter-matrix row of at most kThinGroups * 4 units (256 floats, 512 bfloat16) and at most
// kThinChannels output channels: first layers on camera frames, 1x1 layers on few channels.  The
// tile pipeline above spends most of such a launch filling and draining its ring -- a tile has a
// handful of K slices -- so here a wave works alone: 16 listed positions x 16 channels x the whole
// reduction.  Lane (pixel l % 16, slot l / 16) gathers units slot, 4 + slot, 8 + slot ... of its pixel's
// image-matrix row straight into registers, all loads in flight at once, and feeds them to the
// matrix cores against filter fragments read from an LDS copy of the filter matrix (rows one unit
// apart in the banks).  No barrier after set-up: the three waves of a SIMD hide each other's
// gather latency.  The positions come from the ranked map (each lane finds its own position with
// a binary search over the ranks) or from the list.  Every sum is formed in ascending k by one
// wave, so results do not depend on the number of positions.
static constexpr int kThinGroups = 16;
static constexpr int kThinChannels = 64;
static constexpr int kThinMaxWork = 32;     // groups x channel tiles up to which this kernel is used
static constexpr int kThinWholeFactor = 2; // tiles of 16 positions per wave from which a wave takes all channel tiles
static constexpr int kThinScratchBytes = (2 * kSelMaxWords + 4) * 8;                           // front-end scratch
static constexpr int kThinFilterBytes = kThinChannels * (kThinGroups * 4 + 1) * 16;              // [Mpad][units + 1]
static constexpr int kThinTapBytes = kThinGroups * 4 * (int)sizeof(int2);
static constexpr int kThinSelOffset = kThinScratchBytes + kThinFilterBytes + kThinTapBytes;
static constexpr int kThinSmemBytes = kThinSelOffset + kSelSlots * 12 + 64;
static_assert(kThinSmemBytes <= 160 * 1024, "a workgroup has 160 KiB of LDS");

// The position of rank r (0 <= r < number of selected positions) in a ranked selection map.
__device__ __forceinline__ int select_rank(const Selection &sel, int r)
{
    // the last word whose exclusive rank is <= r holds it: later words start at a higher rank,
    // and of the words sharing its rank it is the last (the others are empty)
    int w = 0;
#pragma unroll
    for (int step = kSelMaxWords; step; step >>= 1)
        if (w + step < sel.nwords && sel.rank[w + step] <= r) w += step;
    const uint64_t bits = sel.words[w];
    int k = r - sel.rank[w], pos = 0; // the k-th set bit of the word, counted from 0
#pragma unroll
    for (int sh = 32; sh; sh >>= 1) {
        const int c = __popcll((bits >> pos) & ((1ull << sh) - 1ull));
        if (k >= c) {
            k -= c;
            pos += sh;
        }
    }
    return w * 64 + pos;
}

// One wave's share of the tiles: 16 positions x TC channel tiles of 16.  In program order per tile:
// find the next tile's positions, multiply the current tile (its gathers were issued a tile ago),
// issue the next tile's gathers into the registers the MFMAs have just read, update the outputs of
// the current tile -- so a tile's gather latency passes during the update before it and the search
// after it.
template <int DT, int TC>
__device__ __forceinline__ void thin_tiles(const GemmArgs &a, const int n, const Selection &sel, const uintx4 *sB,
                                           const int2 *sTap, const int G, const int pitch)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cgroups = (a.Mpad >> 4) / TC; // wave tiles per pixel tile: 1, 2 or 4
    const int cshift = cgroups == 1 ? 0 : (cgroups == 2 ? 1 : 2);
    const long long T = (long long)((n + 15) >> 4) << cshift; // wave tiles, channel group fastest
    const int W = gridDim.x;
    // workgroups are dealt round-robin over the 8 XCDs: number them so that each XCD gets a contiguous range
    const int w = (int)(blockIdx.x & 7) * (W >> 3) + (int)(blockIdx.x >> 3);
    const int t_begin = (int)(T * w / W), t_end = (int)(T * (w + 1) / W);
    const int lrow = lane & 15, lk = lane >> 4;
    const float *x = static_cast<const float *>(a.x);
    const bool detect = a.next_flags != nullptr && !a.next_force;

    struct Where {
        int g, iy0, ix0, base;
    };
    auto locate = [&](int t) {
        const int r = (t >> cshift) * 16 + lrow;
        Where p = {-1, -(1 << 28), -(1 << 28), 0};
        if (r < n) p.g = sel.words ? select_rank(sel, r) : a.list[r];
        if (p.g >= 0) {
            const int st = fast_div(p.g, a.dNo), q = p.g - st * a.No;
            const int qy = fast_div(q, a.dWo), qx = q - qy * a.Wo;
            p.iy0 = qy * a.stride - a.pad;
            p.ix0 = qx * a.stride - a.pad;
            p.base = ((st * a.H + p.iy0) * a.W + p.ix0) * a.pix_words;
        }
        return p;
    };
    floatx4 ra[kThinGroups];
    uintx4 replaced[TC];
    auto gather = [&](const Where &p, int cg) {
#pragma unroll
        for (int gg = 0; gg < kThinGroups; ++gg) {
            if (gg < G) {
                const int2 tp = sTap[4 * gg + lk];
                const int tj = tp.y & 0xff, ti = (tp.y >> 8) & 0xff;
                const bool ok = (tp.y >> 16) != 0 && (unsigned)(p.iy0 + tj) < (unsigned)a.H && (unsigned)(p.ix0 + ti) < (unsigned)a.W;
                // outside the image (or no pixel in this row): the zero unit kept behind the map
                const unsigned idx = ok ? (unsigned)(p.base + tp.x) : (unsigned)a.zero_word;
                ra[gg] = *reinterpret_cast<const floatx4_a4 *>(x + idx);
            }
        }
        // the values about to be replaced, for the change detection of the layer this map feeds
#pragma unroll
        for (int j = 0; j < TC; ++j) {
            const int ch = (cg * TC + j) * 16 + lk * 4;
            replaced[j] = (uintx4){0u, 0u, 0u, 0u};
            if (detect && p.g >= 0 && ch < a.Ms) {
                if constexpr (DT == kBF16) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(static_cast<const unsigned short *>(a.out) + (size_t)p.g * a.Ms + ch);
                    replaced[j][0] = v.x;
                    replaced[j][1] = v.y;
                } else {
                    replaced[j] = *reinterpret_cast<const uintx4 *>(static_cast<const float *>(a.out) + (size_t)p.g * a.Ms + ch);
                }
            }
        }
    };

    int t = t_begin + wave;
    if (t >= t_end) return;
    Where cur = locate(t);
    gather(cur, t & (cgroups - 1));
    while (t < t_end) {
        const int tn = t + NT / 64;
        const bool more = tn < t_end;
        Where nxt = {-1, 0, 0, 0};
        if (more) nxt = locate(tn);
        const int cg = t & (cgroups - 1);
        // MFMA step s of group gg contracts k = 16 gg + 4 slot + s over the four slots (bfloat16: the
        // eight k of a unit at once); D[4 slot + i][pixel] lands in this lane: four consecutive channels
        floatx4 acc[TC];
#pragma unroll
        for (int j = 0; j < TC; ++j) acc[j] = (floatx4){0.f, 0.f, 0.f, 0.f};
        const uintx4 *brow = sB + (cg * TC * 16 + lrow) * pitch + lk;
#pragma unroll
        for (int gg = 0; gg < kThinGroups; ++gg) {
            if (gg < G) {
#pragma unroll
                for (int j = 0; j < TC; ++j) {
                    const uintx4 bq = brow[j * 16 * pitch + 4 * gg];
                    if constexpr (DT == kBF16) {
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bq),
                                                                     __builtin_bit_cast(bf16x8, ra[gg]), acc[j], 0, 0, 0);
                    } else {
                        const floatx4 bf = __builtin_bit_cast(floatx4, bq);
#pragma unroll
                        for (int s = 0; s < 4; ++s) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[s], ra[gg][s], acc[j], 0, 0, 0);
                    }
                }
            }
        }
        uintx4 old[TC];
#pragma unroll
        for (int j = 0; j < TC; ++j) old[j] = replaced[j];
        if (more) gather(nxt, tn & (cgroups - 1));
        // output update: bias, activation, scatter to the stored map
        bool changed = false;
#pragma unroll
        for (int j = 0; j < TC; ++j) {
            const int ch = (cg * TC + j) * 16 + lk * 4;
            if (cur.g >= 0 && ch < a.Ms) {
                const float4 bv = *reinterpret_cast<const float4 *>(a.bias + ch);
                float4 o;
                o.x = acc[j][0] + bv.x;
                o.y = acc[j][1] + bv.y;
                o.z = acc[j][2] + bv.z;
                o.w = acc[j][3] + bv.w;
                if (a.relu) {
                    o.x = fmaxf(o.x, 0.f);
                    o.y = fmaxf(o.y, 0.f);
                    o.z = fmaxf(o.z, 0.f);
                    o.w = fmaxf(o.w, 0.f);
                }
                if constexpr (DT == kBF16) {
                    uint2 nv;
                    nv.x = (unsigned)bf16_bits(o.x) | ((unsigned)bf16_bits(o.y) << 16);
                    nv.y = (unsigned)bf16_bits(o.z) | ((unsigned)bf16_bits(o.w) << 16);
                    if (detect)
                        changed |= fabsf(bf16_value(nv.x & 0xffff) - bf16_value(old[j][0] & 0xffff)) > a.next_tau ||
                                   fabsf(bf16_value(nv.x >> 16) - bf16_value(old[j][0] >> 16)) > a.next_tau ||
                                   fabsf(bf16_value(nv.y & 0xffff) - bf16_value(old[j][1] & 0xffff)) > a.next_tau ||
                                   fabsf(bf16_value(nv.y >> 16) - bf16_value(old[j][1] >> 16)) > a.next_tau;
                    *reinterpret_cast<uint2 *>(static_cast<unsigned short *>(a.out) + (size_t)cur.g * a.Ms + ch) = nv;
                } else {
                    if (detect)
                        changed |= fabsf(o.x - __uint_as_float(old[j][0])) > a.next_tau ||
                                   fabsf(o.y - __uint_as_float(old[j][1])) > a.next_tau ||
                                   fabsf(o.z - __uint_as_float(old[j][2])) > a.next_tau ||
                                   fabsf(o.w - __uint_as_float(old[j][3])) > a.next_tau;
                    *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + (size_t)cur.g * a.Ms + ch) = o;
                }
            }
        }
        if (a.next_flags) {
            int f = a.next_force ? 1 : (int)changed;
            // the other channels of this pixel sit in the lanes 16, 32 and 48 further on
            f |= __shfl_xor(f, 16);
            f |= __shfl_xor(f, 32);
            if (lk == 0 && f && cur.g >= 0) a.next_flags[cur.g] = 1;
        }
        cur = nxt;
        t = tn;
    }
}

// MT: channel tiles of the layer (Mpad / 16).  A wave takes all of them for its 16 positions when
// there are enough positions to occupy every wave that way, else one each.
template <int DT, int MT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu((NT + 255) / 256, (NT + 255) / 256))) void gemm_thin_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) float smem[];
    char *lds = reinterpret_cast<char *>(smem);
    uintx4 *sB = reinterpret_cast<uintx4 *>(lds + kThinScratchBytes);
    int2 *sTap = reinterpret_cast<int2 *>(lds + kThinScratchBytes + kThinFilterBytes);
    const int tid = threadIdx.x;
    const int nu = a.Kpad / Unit<DT>::N; // units per filter-matrix row: a multiple of eight
    const int G = nu >> 2, pitch = nu + 1;
    {
        const uintx4 *wt = static_cast<const uintx4 *>(a.wt);
        for (int i = tid; i < a.Mpad * nu; i += NT) {
            const int r = fast_div(i >> 3, a.dNk), u = i - r * nu;
            sB[r * pitch + u] = wt[i];
        }
        for (int i = tid; i < nu; i += NT) sTap[i] = a.taps[i];
    }
    Selection sel = {nullptr, nullptr, 0};
    int n;
    if (a.sel_words > 0) {
        uint64_t *sW = reinterpret_cast<uint64_t *>(lds + kThinSelOffset);
        int *sRank = reinterpret_cast<int *>(lds + kThinSelOffset + kSelSlots * 8);
        n = rank_selection(a, sW, sRank, sRank + kSelSlots, reinterpret_cast<uint64_t *>(lds));
        sel.words = sW;
        sel.rank = sRank;
        sel.nwords = a.sel_words;
    } else {
        n = *a.count;
    }
    __syncthreads();
    if constexpr (MT > 1) {
        if (((n + 15) >> 4) >= kThinWholeFactor * (NT / 64) * (int)gridDim.x) {
            thin_tiles<DT, MT>(a, n, sel, sB, sTap, G, pitch);
            return;
        }
    }
    thin_tiles<DT, 1>(a, n, sel, sB, sTap, G, pitch);
}

// Measured against the tile pipeline on 3..256 input and 8..64 output channels, 4 800 to 4 million
// positions: the lone waves win as long as (groups of four units) x (channel tiles) stays at or
// below 32 -- beyond that a wave's chain of MFMAs per tile gets long and the big tiles' reuse of
// filter fragments pays.
static bool gemm_is_thin(const GemmArgs &a)
{
    const int nu = a.Kpad / elems_per_unit(a.dtype);
    return nu <= kThinGroups * 4 && (a.Mpad == 16 || a.Mpad == 32 || a.Mpad == 64) && (nu / 4) * (a.Mpad / 16) <= kThinMaxWork;
}

// ---- host side --------------------------------------------------------------------------
int gemm_k_multiple(int dtype) { return BK * 4 / elem_bytes(dtype); }

void gemm_set_divisors(GemmArgs &a)
{
    a.dNo = make_fastdiv(a.No > 0 ? a.No : 1);
    a.dWo = make_fastdiv(a.Wo > 0 ? a.Wo : 1);
    a.dHo = make_fastdiv(a.Wo > 0 && a.No >= a.Wo ? a.No / a.Wo : 1);
    const int nk = a.Kpad / gemm_k_multiple(a.dtype);
    a.dNk = make_fastdiv(nk > 0 ? nk : 1);
    a.dGrid = make_fastdiv(a.grid > 0 ? a.grid : 1);
    a.dVin = make_fastdiv(a.pix_words > 0 ? (a.pix_words + 3) / 4 : 1);
    a.dKw = make_fastdiv(a.kw > 0 ? a.kw : 1);
}

int gemm_select_max_words(void) { return kSelMaxWords; }

int gemm_channel_tile(int M)
{
    if (M <= 16) return 16;
    if (M <= 32) return 32;
    if (M <= 64) return 64;
    return 128;
}

// Pixels per big tile.  The 64-channel kernel takes 128 instead of 256 on maps of at most
// kNarrowTilePixels positions, where a 256-pixel tile would leave most workgroups a third of a tile's K
// range (16->64 7x7: 35.5 -> 33.6 us at 160x120, but 230 -> 248 us at 640x360).
static constexpr int kNarrowTilePixels = 65536;
static int pixel_tile(int bm, int max_pixels)
{
    if (bm == 128) return 128;
    return bm == 64 && max_pixels <= kNarrowTilePixels ? 128 : 256;
}

// Two partial-accumulator slabs per workgroup.
size_t gemm_partial_bytes(int M, int grid)
{
    const int bm = gemm_channel_tile(M);
    return (size_t)2 * grid * bm * pixel_tile(bm, 0x7fffffff) * sizeof(float); // the widest tile of that channel tile
}

// One ticket counter per shared tile (fewer than the workgroup count); zero between launches.
size_t gemm_ticket_bytes(int grid) { return (size_t)grid * sizeof(int); }

// Workgroups to launch: one per compute unit, fewer if even the longest list gives less work.
int gemm_grid(const GemmArgs &a, int compute_units)
{
    const int bm = gemm_channel_tile(a.M), bn = pixel_tile(bm, a.max_pixels);
    int W = compute_units & ~7;
    if (W < 8) W = 8;
    if (W > kMaxGrid) W = kMaxGrid;
    if (gemm_is_thin(a)) {
        // a workgroup per four wave tiles of 16 positions x 16 channels (one per SIMD: spreading a short
        // list over more compute units shortens the launch, 128->16 1x1 at 160x120: 6.6 -> 5.4 us)
        const long long wave_tiles = (long long)((a.max_pixels + 15) / 16) * (a.Mpad / 16);
        long long need = ((wave_tiles + 3) / 4 + 7) / 8 * 8;
        if (need < 8) need = 8;
        return (int)(need < W ? need : W);
    }
    const int nk = a.Kpad / gemm_k_multiple(a.dtype);
    const int parts = nk / kMinIters > 1 ? nk / kMinIters : 1;
    // with few pixels the small tile (64 pixels) is used: count those
    const long long big = (long long)((a.max_pixels + bn - 1) / bn) * (a.Mpad / bm);
    const long long tiles = big * kSmallTileFactor >= W ? big : (long long)((a.max_pixels + 63) / 64) * (a.Mpad / bm);
    long long need = tiles >= W ? W : (tiles * parts + 7) / 8 * 8;
    if (need < 8) need = 8;
    return (int)(need < W ? need : W);
}

// BM; big tile (BN, WM, WN, ring slices, direct-to-LDS producers); small tile (the same)
#define CBK_VARIANTS(X)                                         \
    X(16, 256, 1, 8, 3, false, 128, 1, 8, 3, false)             \
    X(32, 256, 1, 8, 3, false, 64, 2, 4, 3, false)              \
    X(64, 256, 2, 4, 3, false, 64, 2, 4, 3, false)              \
    X(64, 128, 2, 4, 3, false, 64, 2, 4, 3, false)              \
    X(128, 128, 2, 4, 4, true, 64, 4, 2, 5, true)

hipError_t gemm_prepare(void)
{
    hipError_t e = hipSuccess;
#define X(BM_, BNB_, WMB_, WNB_, SB_, DB_, BNS_, WMS_, WNS_, SS_, DS_)                                                        \
    if (e == hipSuccess)                                                                                                      \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(                                                               \
                                    &gemm_gather_kernel<kF32, BM_, BNB_, WMB_, WNB_, SB_, DB_, BNS_, WMS_, WNS_, SS_, DS_>),   \
                                hipFuncAttributeMaxDynamicSharedMemorySize, KernelSmem<BM_, BNB_, SB_, BNS_, SS_>::bytes);    \
    if (e == hipSuccess)                                                                                                      \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(                                                               \
                                    &gemm_gather_kernel<kBF16, BM_, BNB_, WMB_, WNB_, SB_, DB_, BNS_, WMS_, WNS_, SS_, DS_>),  \
                                hipFuncAttributeMaxDynamicSharedMemorySize, KernelSmem<BM_, BNB_, SB_, BNS_, SS_>::bytes);
    CBK_VARIANTS(X)
#undef X
#define T(DT_, MT_)                                                                                                \
    if (e == hipSuccess)                                                                                           \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_thin_kernel<DT_, MT_>),                       \
                                hipFuncAttributeMaxDynamicSharedMemorySize, kThinSmemBytes);
    T(kF32, 1) T(kF32, 2) T(kF32, 4) T(kBF16, 1) T(kBF16, 2) T(kBF16, 4)
#undef T
    return e;
}

template <int BM, int BNB, int WMB, int WNB, int SB, bool DB, int BNS, int WMS, int WNS, int SS, bool DS>
static hipError_t launch(hipStream_t st, const GemmArgs &a, const Timing &tm)
{
    constexpr int smem_bytes = KernelSmem<BM, BNB, SB, BNS, SS>::bytes;
    if (a.dtype == kBF16)
        launch_kernel(tm, gemm_gather_kernel<kBF16, BM, BNB, WMB, WNB, SB, DB, BNS, WMS, WNS, SS, DS>, dim3(a.grid),
                      dim3(NT), smem_bytes, st, a);
    else
        launch_kernel(tm, gemm_gather_kernel<kF32, BM, BNB, WMB, WNB, SB, DB, BNS, WMS, WNS, SS, DS>, dim3(a.grid),
                      dim3(NT), smem_bytes, st, a);
    return hipGetLastError();
}

hipError_t gemm_gather(hipStream_t st, const GemmArgs &a, const Timing &tm)
{
    const int bm = gemm_channel_tile(a.M), bn = pixel_tile(bm, a.max_pixels);
    const int eu = elems_per_unit(a.dtype);
    if (a.Mpad % bm != 0 || a.Kpad % gemm_k_multiple(a.dtype) != 0 || a.Ms % eu != 0 || a.pix_words < 1 || !a.partial ||
        !a.tickets || a.grid < 8 || (a.grid & 7) || a.grid > kMaxGrid)
        return hipErrorInvalidValue;
    // the direct-to-LDS producers address a channel tile's filter rows with 32-bit byte offsets
    if ((long long)bm * a.Kpad * 4 >= (1ll << 32)) return hipErrorInvalidValue;
    // the divisors must belong to these arguments, and the schedule's 32-bit arithmetic must hold
    if (a.kh < 1 || a.kw < 1 || a.dKw.d != a.kw || a.dVin.d != (a.pix_words + 3) / 4) return hipErrorInvalidValue;
    if (a.dNo.d != a.No || a.dWo.d != a.Wo || a.dHo.d * a.Wo != a.No || a.dGrid.d != a.grid ||
        a.dNk.d != a.Kpad / gemm_k_multiple(a.dtype) || a.dNk.d >= (1 << 20))
        return hipErrorInvalidValue;
    if (a.sel_words > 0 && a.sel_dilate &&
        (a.stride != 1 || a.kw > 16 || a.kw < 1 || a.kh < 1 || a.kh > 16 || !a.upd_out || a.S < 1 || a.sel_in_words < 1 ||
         a.sel_in_words > kSelMaxWords || ((long long)a.S * a.H * a.Wo + 63) / 64 > kSelMaxWords ||
         (long long)a.sel_in_words * 64 < (long long)a.S * a.N || a.No % a.Wo != 0))
        return hipErrorInvalidValue;
    if (a.sel_words < 0 || a.sel_words > kSelMaxWords || (a.sel_words > 0 && !a.sel_map) ||
        (a.sel_words == 0 && (!a.list || !a.count)) || (long long)a.sel_words * 64 < a.max_pixels * (a.sel_words > 0))
        return hipErrorInvalidValue;
    if (gemm_is_thin(a)) {
#define T(DT_, MT_)                                                                                      \
    if (a.dtype == DT_ && a.Mpad == 16 * MT_) {                                                           \
        launch_kernel(tm, gemm_thin_kernel<DT_, MT_>, dim3(a.grid), dim3(NT), kThinSmemBytes, st, a);    \
        return hipGetLastError();                                                                        \
    }
        T(kF32, 1) T(kF32, 2) T(kF32, 4) T(kBF16, 1) T(kBF16, 2) T(kBF16, 4)
#undef T
    }
#define X(BM_, BNB_, WMB_, WNB_, SB_, DB_, BNS_, WMS_, WNS_, SS_, DS_) \
    if (bm == BM_ && bn == BNB_) return launch<BM_, BNB_, WMB_, WNB_, SB_, DB_, BNS_, WMS_, WNS_, SS_, DS_>(st, a, tm);
    CBK_VARIANTS(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace cbk
