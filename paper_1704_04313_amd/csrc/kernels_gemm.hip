// Gathered matrix generation + matrix multiplication + output update for gfx950.
//
// Section 3.1 of the paper assembles only the columns of the image matrix X that belong to
// output positions needing an update, multiplies them with the unchanged filter matrix K and
// writes the result (with the activation) over the stored output.  Here matrix generation and
// multiplication are one kernel: a workgroup owns BN listed output positions x BM output
// channels and builds the BN x 32 slices of the reduced X directly in LDS by gathering 16-byte
// channel groups from the channel-contiguous input map; the reduced X never exists in HBM.
//
// The workgroup has eight waves with two roles.  Waves 4-7 ("producers") compute gather
// addresses, load the next K slice of both operands from global memory and store it to LDS;
// waves 0-3 ("consumers") only read LDS fragments and issue v_mfma_f32_16x16x4_f32 (fp32 in,
// fp32 accumulate).  One producer and one consumer wave share each SIMD, so address
// arithmetic, global-load latency and LDS stores overlap the matrix pipeline instead of
// draining it once per slice.
#include "kernels.h"

#include <cstdio>
#include <cstdlib>

namespace cbk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

static constexpr int BK = 32;       // K slice per pipeline stage (floats)
static constexpr int LDK = BK + 4;  // LDS row pitch: 36 floats keeps 16-byte alignment and makes
                                    // the rows read by one ds_read_b128 phase hit distinct banks
static constexpr int NT = 512;      // threads per workgroup: 4 consumer + 4 producer waves
static constexpr int NPROD = 256;   // producer threads
static constexpr int kMaxSplit = 16;   // deepest K split
static constexpr int kMaxItems = 1024; // most work items a split multiplication may create
static constexpr int kCUs = 256;       // compute units of an MI355X; one workgroup each
static constexpr int kStages = 3;      // K slices resident in LDS

template <int BM, int BN>
struct TileSmem {
    static constexpr int a_floats = BN * LDK;
    static constexpr int b_floats = BM * LDK;
    static constexpr int bytes = kStages * (a_floats + b_floats) * 4 + BN * 4;
};

// How many K ranges a tile's contraction is split into.  A function of the tile count and
// the K length only, so that the multiplication kernel and the output-update kernel (and two
// runs on the same input) always agree.  With few listed pixels there are too few tiles to
// occupy 256 compute units; splitting K restores the parallelism at the price of writing
// partial sums that the output update adds up in a fixed order (deterministic results).
// Picks the split with the least (rounds over the compute units) x (slices per item + fixed
// cost of starting and finishing an item).
__host__ __device__ inline int choose_split(int tiles, int nk, int split_override)
{
    int smax = nk / 4;
    if (smax > kMaxSplit) smax = kMaxSplit;
    if (smax < 1) smax = 1;
    if (tiles < 1) return 1;
    int best = 1;
    if (split_override > 0) {
        best = split_override < smax ? split_override : smax;
    } else {
        if (tiles >= 4 * kCUs) return 1;
        long long best_cost = -1;
        for (int s = 1; s <= smax; ++s) {
            const long long rounds = ((long long)tiles * s + kCUs - 1) / kCUs;
            const long long cost = rounds * ((nk + s - 1) / s + 2);
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                best = s;
            }
        }
    }
    while (best > 1 && (long long)best * tiles > kMaxItems) --best;
    return best;
}

// Image-matrix rows gathered by one producer thread for one K slice: PA rows (32 apart), one
// float4 each.  tp is the slice's tap descriptor for this thread's float4 column.
template <int PA>
__device__ __forceinline__ void gather_rows(const GemmArgs &a, const int2 tp, const int (&iy0)[PA],
                                            const int (&ix0)[PA], const int (&base)[PA], floatx4 (&ra)[PA])
{
    const int tj = tp.y & 0xff, ti = (tp.y >> 8) & 0xff;
    const bool tv = (tp.y >> 16) != 0;
#pragma unroll
    for (int ps = 0; ps < PA; ++ps) {
        const bool ok = tv && (unsigned)(iy0[ps] + tj) < (unsigned)a.H && (unsigned)(ix0[ps] + ti) < (unsigned)a.W;
        ra[ps] = ok ? *reinterpret_cast<const floatx4 *>(a.x + (base[ps] + tp.x)) : (floatx4){0.f, 0.f, 0.f, 0.f};
    }
}

template <int BM, int PB>
__device__ __forceinline__ void load_filter_rows(const float *wrow, int kpad, int kc, int r0, floatx4 (&rb)[PB])
{
    if constexpr (BM >= 32) {
#pragma unroll
        for (int ps = 0; ps < PB; ++ps)
            rb[ps] = *reinterpret_cast<const floatx4 *>(wrow + (size_t)(32 * ps) * kpad + kc * BK);
    } else {
        if (r0 < BM) rb[0] = *reinterpret_cast<const floatx4 *>(wrow + kc * BK);
    }
}

template <int BM, int PA, int PB>
__device__ __forceinline__ void stage_rows(float *A, float *B, int r0, int v, const floatx4 (&ra)[PA],
                                           const floatx4 (&rb)[PB])
{
#pragma unroll
    for (int ps = 0; ps < PA; ++ps) *reinterpret_cast<floatx4 *>(A + (r0 + 32 * ps) * LDK + v * 4) = ra[ps];
    if constexpr (BM >= 32) {
#pragma unroll
        for (int ps = 0; ps < PB; ++ps) *reinterpret_cast<floatx4 *>(B + (r0 + 32 * ps) * LDK + v * 4) = rb[ps];
    } else {
        if (r0 < BM) *reinterpret_cast<floatx4 *>(B + r0 * LDK + v * 4) = rb[0];
    }
}

// BM x BN workgroup tile; the four consumer waves are arranged WM (channels) x WN (pixels).
//
// LDS holds a ring of three K slices.  In iteration kc the producers store slice kc+2 and issue
// the global loads of slice kc+3, while the consumers multiply slice kc and already read the
// first fragments of slice kc+1, so the matrix pipeline keeps running across the one barrier
// per slice.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_gather_kernel(GemmArgs a)
{
    static_assert(WM * WN == 4, "four consumer waves");
    constexpr int TP = BN / WN / 16; // 16-pixel MFMA tiles per consumer wave
    constexpr int TC = BM / WM / 16; // 16-channel MFMA tiles per consumer wave
    constexpr int PA = BN / 32;      // image-matrix rows staged per producer thread and slice
    constexpr int PB = (BM + 31) / 32;
    constexpr int ASZ = BN * LDK, BSZ = BM * LDK;
    static_assert(TP >= 1 && TC >= 1, "tile too small");
    static_assert(BK == 32, "two 16-wide fragment groups per slice");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                                    // [3][BN][LDK]  gathered image-matrix slices
    float *Bs = smem + kStages * ASZ;                    // [3][BM][LDK]  filter-matrix slices
    int *sU = reinterpret_cast<int *>(Bs + kStages * BSZ); // [BN] listed pixels of this tile (-1: none)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const bool producer = wave >= 4;

    const int n = *a.count;
    const int mtiles = a.Mpad / BM;
    const int ptiles = (n + BN - 1) / BN;
    const int nk = a.Kpad / BK;
    const int S = choose_split(ptiles * mtiles, nk, a.split_override);
    const int items = ptiles * mtiles * S;
    // Consecutive work items share their gathered pixels (channel tiles of one pixel tile) or
    // their filter slice; give each XCD (workgroups are dealt round-robin over the 8 XCDs) one
    // contiguous range of items so that this sharing happens inside one L2.
    const int per_xcd = (items + 7) / 8;

    for (int b = blockIdx.x; b < per_xcd * 8; b += gridDim.x) {
        const int item = (b & 7) * per_xcd + (b >> 3);
        if (item >= items) continue;
        const int mt = item % mtiles;
        const int ks = (item / mtiles) % S;
        const int pt = item / (mtiles * S);
        const int kc0 = (int)((long long)ks * nk / S);
        const int kc1 = (int)((long long)(ks + 1) * nk / S);

        __syncthreads(); // the previous item's LDS reads are done
        for (int i = tid; i < BN; i += NT) {
            const int u = pt * BN + i;
            sU[i] = (u < n) ? a.list[u] : -1;
        }
        __syncthreads();

        // Both roles execute the same number of barriers: one after the prologue and one per slice.
        if (producer) {
            const int ptid = tid & (NPROD - 1);
            const int v = ptid & 7;   // float4 column inside the K slice
            const int r0 = ptid >> 3; // first row this thread stages
            int iy0[PA], ix0[PA], base[PA];
#pragma unroll
            for (int ps = 0; ps < PA; ++ps) {
                const int g = sU[r0 + 32 * ps];
                if (g >= 0) {
                    const int st = g / a.No, q = g - st * a.No;
                    const int qy = q / a.Wo, qx = q - qy * a.Wo;
                    iy0[ps] = qy * a.stride - a.pad;
                    ix0[ps] = qx * a.stride - a.pad;
                    base[ps] = ((st * a.H + iy0[ps]) * a.W + ix0[ps]) * a.Cs;
                } else {
                    iy0[ps] = -(1 << 28);
                    ix0[ps] = -(1 << 28);
                    base[ps] = 0;
                }
            }
            const float *wrow = a.wt + (size_t)(mt * BM + r0) * a.Kpad + v * 4;
            const int2 *taps = a.taps + v;
            floatx4 ra[PA], rb[PB], ra2[PA], rb2[PB];
            // prologue: slices kc0 and kc0+1 into ring slots 0 and 1, slice kc0+2 into registers
            const int2 t0 = taps[kc0 * (BK / 4)];
            const int2 t1 = taps[(kc0 + 1 < kc1 ? kc0 + 1 : kc0) * (BK / 4)];
            int2 tp = taps[(kc0 + 2 < kc1 ? kc0 + 2 : kc0) * (BK / 4)];
            gather_rows<PA>(a, t0, iy0, ix0, base, ra);
            load_filter_rows<BM, PB>(wrow, a.Kpad, kc0, r0, rb);
            if (kc0 + 1 < kc1) {
                gather_rows<PA>(a, t1, iy0, ix0, base, ra2);
                load_filter_rows<BM, PB>(wrow, a.Kpad, kc0 + 1, r0, rb2);
            }
            stage_rows<BM, PA, PB>(As, Bs, r0, v, ra, rb);
            if (kc0 + 1 < kc1) stage_rows<BM, PA, PB>(As + ASZ, Bs + BSZ, r0, v, ra2, rb2);
            if (kc0 + 2 < kc1) {
                gather_rows<PA>(a, tp, iy0, ix0, base, ra);
                load_filter_rows<BM, PB>(wrow, a.Kpad, kc0 + 2, r0, rb);
                if (kc0 + 3 < kc1) tp = taps[(kc0 + 3) * (BK / 4)];
            }
            __syncthreads();
            int slot = 2; // ring slot of slice kc+2
            for (int kc = kc0; kc < kc1; ++kc) {
#ifdef CBK_EXP_NOPRODUCER
                if (false) {
#else
                if (kc + 2 < kc1) {
#endif
                    stage_rows<BM, PA, PB>(As + slot * ASZ, Bs + slot * BSZ, r0, v, ra, rb);
                    if (kc + 3 < kc1) {
                        gather_rows<PA>(a, tp, iy0, ix0, base, ra);
                        load_filter_rows<BM, PB>(wrow, a.Kpad, kc + 3, r0, rb);
                        if (kc + 4 < kc1) tp = taps[(kc + 4) * (BK / 4)];
                    }
                }
                slot = slot == kStages - 1 ? 0 : slot + 1;
#ifndef CBK_EXP_NOBARRIER
                __syncthreads();
#endif
            }
        } else {
            const int wpx0 = (wave % WN) * (BN / WN);
            const int wch0 = (wave / WN) * (BM / WM);
            const int lrow = lane & 15; // row of the 16-row operand tiles this lane feeds
            const int lk = lane >> 4;   // k slot this lane feeds
            floatx4 acc[TC][TP];
#pragma unroll
            for (int j = 0; j < TC; ++j)
#pragma unroll
                for (int i = 0; i < TP; ++i) acc[j][i] = (floatx4){0.f, 0.f, 0.f, 0.f};
            const float *A0 = As + (wpx0 + lrow) * LDK + lk * 4;
            const float *B0 = Bs + (wch0 + lrow) * LDK + lk * 4;
            // Each lane reads four consecutive k of its row; MFMA step s then contracts
            // k = 16*group + 4*slot + s for slot = 0..3 -- both operands use the same permutation.
            // D = (filter rows) x (pixel columns): D[4*slot + r][lane%16] lands in this lane,
            // i.e. four consecutive channels of one pixel per accumulator.
            floatx4 af[2][TP], bf[2][TC];
            auto read_frags = [&](int set, int slot, int kk) {
                const float *A = A0 + slot * ASZ + kk * 16;
                const float *B = B0 + slot * BSZ + kk * 16;
#pragma unroll
                for (int i = 0; i < TP; ++i) af[set][i] = *reinterpret_cast<const floatx4 *>(A + i * 16 * LDK);
#pragma unroll
                for (int j = 0; j < TC; ++j) bf[set][j] = *reinterpret_cast<const floatx4 *>(B + j * 16 * LDK);
            };
            auto multiply = [&](int set) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int j = 0; j < TC; ++j)
#pragma unroll
                        for (int i = 0; i < TP; ++i)
                            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[set][j][s], af[set][i][s], acc[j][i],
                                                                             0, 0, 0);
            };
            __syncthreads();
            read_frags(0, 0, 0);
            int slot = 0; // ring slot of slice kc
            for (int kc = kc0; kc < kc1; ++kc) {
                const int nslot = slot == kStages - 1 ? 0 : slot + 1;
                // The scheduling barriers pin the order "issue the LDS reads of the next fragment
                // group, then the 64 MFMAs of the current one", so that LDS latency and bandwidth
                // are spent while the matrix pipeline is busy.
#ifndef CBK_EXP_NOLDSREAD
                read_frags(1, slot, 1);
#endif
                __builtin_amdgcn_sched_barrier(0);
                multiply(0);
                __builtin_amdgcn_sched_barrier(0);
#ifndef CBK_EXP_NOLDSREAD
                if (kc + 1 < kc1) read_frags(0, nslot, 0);
#endif
                __builtin_amdgcn_sched_barrier(0);
                multiply(1);
                __builtin_amdgcn_sched_barrier(0);
                slot = nslot;
#ifndef CBK_EXP_NOBARRIER
                __syncthreads();
#endif
            }

            if (S == 1) {
                // Output update fused: bias, activation, scatter to the stored map.
#pragma unroll
                for (int j = 0; j < TC; ++j) {
                    const int ch = mt * BM + wch0 + j * 16 + lk * 4;
                    const float4 bv = *reinterpret_cast<const float4 *>(a.bias + ch);
#pragma unroll
                    for (int i = 0; i < TP; ++i) {
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
                            *reinterpret_cast<float4 *>(a.out + (size_t)g * a.Ms + ch) = o;
                        }
                    }
                }
            } else {
                // Partial sums of this K range, [pixel][channel] inside the item's slab.
                float *slab = a.partial + (size_t)item * (BN * BM);
#pragma unroll
                for (int j = 0; j < TC; ++j)
#pragma unroll
                    for (int i = 0; i < TP; ++i) {
                        float4 o;
                        o.x = acc[j][i][0];
                        o.y = acc[j][i][1];
                        o.z = acc[j][i][2];
                        o.w = acc[j][i][3];
                        *reinterpret_cast<float4 *>(slab + (wpx0 + i * 16 + lrow) * BM + wch0 + j * 16 + lk * 4) = o;
                    }
            }
        }
    }
}

// Output update after a split multiplication (Section 3.1, "Output Updating"): add the K-range
// partial sums in ascending K order, add the bias, apply the activation and write the listed
// positions of the stored map.  One thread per (listed pixel, 4 channels): reads and writes are
// contiguous runs of 16*Ms/4 bytes per pixel.  Does nothing if the multiplication was not split.
template <int BM, int BN>
__global__ __launch_bounds__(256) void output_update_kernel(GemmArgs a)
{
    const int n = *a.count;
    const int mtiles = a.Mpad / BM;
    const int ptiles = (n + BN - 1) / BN;
    const int S = choose_split(ptiles * mtiles, a.Kpad / BK, a.split_override);
    if (S == 1) return;
    const int V = a.Ms >> 2;
    const long long total = (long long)n * V;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
        const int u = (int)(idx / V);
        const int ch = (int)(idx - (long long)u * V) * 4;
        const int pt = u / BN, pl = u - pt * BN;
        const int mt = ch / BM, cl = ch - mt * BM;
        const float *p = a.partial + ((size_t)(pt * S) * mtiles + mt) * (BN * BM) + (size_t)pl * BM + cl;
        float4 sum = *reinterpret_cast<const float4 *>(p);
        for (int s = 1; s < S; ++s) {
            const float4 t = *reinterpret_cast<const float4 *>(p + (size_t)s * mtiles * (BN * BM));
            sum.x += t.x;
            sum.y += t.y;
            sum.z += t.z;
            sum.w += t.w;
        }
        const float4 bv = *reinterpret_cast<const float4 *>(a.bias + ch);
        sum.x += bv.x;
        sum.y += bv.y;
        sum.z += bv.z;
        sum.w += bv.w;
        if (a.relu) {
            sum.x = fmaxf(sum.x, 0.f);
            sum.y = fmaxf(sum.y, 0.f);
            sum.z = fmaxf(sum.z, 0.f);
            sum.w = fmaxf(sum.w, 0.f);
        }
        *reinterpret_cast<float4 *>(a.out + (size_t)a.list[u] * a.Ms + ch) = sum;
    }
}

// ---- host side --------------------------------------------------------------------------
int gemm_k_multiple(void) { return BK; }

int gemm_channel_tile(int M)
{
    if (M <= 16) return 16;
    if (M <= 32) return 32;
    if (M <= 64) return 64;
    return 128;
}

static int pixel_tile(int bm) { return bm == 128 ? 128 : 256; }

size_t gemm_partial_bytes(int M)
{
    const int bm = gemm_channel_tile(M);
    return (size_t)kMaxItems * bm * pixel_tile(bm) * sizeof(float);
}

#define CBK_VARIANTS(X) X(16, 256, 1, 4) X(32, 256, 1, 4) X(64, 256, 1, 4) X(128, 128, 2, 2)

hipError_t gemm_prepare(void)
{
    hipError_t e = hipSuccess;
#define X(BM_, BN_, WM_, WN_)                                                                            \
    if (e == hipSuccess)                                                                                 \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_gather_kernel<BM_, BN_, WM_, WN_>), \
                                hipFuncAttributeMaxDynamicSharedMemorySize, TileSmem<BM_, BN_>::bytes);
    CBK_VARIANTS(X)
#undef X
    if (getenv("CBINFER_DEBUG")) {
#define X(BM_, BN_, WM_, WN_)                                                                              \
    {                                                                                                      \
        int nb = -1;                                                                                       \
        (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(                                                \
            &nb, reinterpret_cast<const void *>(&gemm_gather_kernel<BM_, BN_, WM_, WN_>), NT,              \
            TileSmem<BM_, BN_>::bytes);                                                                    \
        fprintf(stderr, "gemm_gather<%d,%d>: %d B LDS, %d workgroups/CU\n", BM_, BN_,                       \
                (int)TileSmem<BM_, BN_>::bytes, nb);                                                       \
    }
        CBK_VARIANTS(X)
#undef X
    }
    return e;
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch(hipStream_t st, const GemmArgs &a)
{
    constexpr int smem_bytes = TileSmem<BM, BN>::bytes;
    gemm_gather_kernel<BM, BN, WM, WN><<<dim3(a.grid), dim3(NT), smem_bytes, st>>>(a);
    return hipGetLastError();
}

template <int BM, int BN>
static hipError_t launch_update(hipStream_t st, const GemmArgs &a)
{
    // has work only while the tile count is below the splitting limit
    long long work = (long long)4 * kCUs * BN * (a.Ms / 4);
    const long long full = (long long)a.max_pixels * (a.Ms / 4);
    if (full < work) work = full;
    long long grid = (work + 255) / 256;
    if (grid > 2048) grid = 2048;
    if (grid < 1) grid = 1;
    output_update_kernel<BM, BN><<<dim3((int)grid), dim3(256), 0, st>>>(a);
    return hipGetLastError();
}

// Workgroups to launch: the largest work-item count any list length can produce, capped.
int gemm_grid(const GemmArgs &a)
{
    const int bm = gemm_channel_tile(a.M), bn = pixel_tile(bm);
    const int nk = a.Kpad / BK, mtiles = a.Mpad / bm;
    const int maxpt = (a.max_pixels + bn - 1) / bn;
    long long best = 1;
    for (int pt = 1; pt <= maxpt; ++pt) {
        const long long t = (long long)pt * mtiles;
        const long long items = t * choose_split((int)(t > 0x7fffffff ? 0x7fffffff : t), nk, a.split_override);
        if (items > best) best = items;
        if (best >= 1024) break;
    }
    if (best > 1024) best = 1024;
    return (int)((best + 7) / 8 * 8);
}

bool gemm_can_split(const GemmArgs &a) { return choose_split(1, a.Kpad / BK, a.split_override) > 1; }

hipError_t gemm_gather(hipStream_t st, const GemmArgs &a)
{
    const int bm = gemm_channel_tile(a.M);
    if (a.Mpad % bm != 0 || a.Kpad % BK != 0 || a.Cs % 4 != 0 || !a.partial || a.grid < 1)
        return hipErrorInvalidValue;
    switch (bm) {
    case 16: return launch<16, 256, 1, 4>(st, a);
    case 32: return launch<32, 256, 1, 4>(st, a);
    case 64: return launch<64, 256, 1, 4>(st, a);
    default: return launch<128, 128, 2, 2>(st, a);
    }
}

hipError_t output_update(hipStream_t st, const GemmArgs &a)
{
    const int bm = gemm_channel_tile(a.M);
    switch (bm) {
    case 16: return launch_update<16, 256>(st, a);
    case 32: return launch_update<32, 256>(st, a);
    case 64: return launch_update<64, 256>(st, a);
    default: return launch_update<128, 128>(st, a);
    }
}

} // namespace cbk
