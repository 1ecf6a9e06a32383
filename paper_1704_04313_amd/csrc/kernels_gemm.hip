// Gathered matrix generation + matrix multiplication + output update for gfx950.
//
// Section 3.1 of the paper assembles only the columns of the image matrix X that belong to
// output positions needing an update, multiplies them with the unchanged filter matrix K and
// writes the result (with the activation) over the stored output.  Here the three steps are
// one kernel: a workgroup owns BN listed output positions x BM output channels, builds the
// BN x 32 slices of the reduced X directly in LDS by gathering 16-byte channel groups from the
// channel-contiguous input map, multiplies on the matrix cores (v_mfma_f32_16x16x4_f32,
// fp32 in, fp32 accumulate) and scatters bias + ReLU results straight to the stored map.
// The reduced X never exists in HBM.
#include "kernels.h"

namespace cbk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

static constexpr int BK = 32;       // K slice per pipeline stage (floats)
static constexpr int LDK = BK + 4;  // LDS row pitch: 36 floats keeps 16-byte alignment and makes
                                    // the 16 rows read by one ds_read_b128 phase hit distinct banks
static constexpr int NT = 256;      // threads per workgroup (4 waves)
static constexpr int kMaxSplit = 16;   // deepest K split
static constexpr int kMaxItems = 1024; // most work items a split multiplication may create

template <int BM, int BN>
struct TileSmem {
    static constexpr int a_floats = BN * LDK;
    static constexpr int b_floats = BM * LDK;
    static constexpr int bytes = 2 * (a_floats + b_floats) * 4 + BN * 4;
};

// How many K ranges a tile's contraction is split into.  A function of the tile count and
// the K length only, so that the multiplication kernel and the output-update kernel (and two
// runs on the same input) always agree.  With few listed pixels there are too few tiles to
// occupy 256 compute units; splitting K restores the parallelism at the price of writing
// partial sums that the output update adds up in a fixed order (deterministic results).
__host__ __device__ inline int choose_split(int tiles, int nk, int split_override)
{
    int smax = nk / 4;
    if (smax > kMaxSplit) smax = kMaxSplit;
    if (smax < 1) smax = 1;
    int s;
    if (split_override > 0) {
        s = split_override;
    } else {
        if (tiles >= 384 || tiles < 1) return 1;
        s = (512 + tiles / 2) / tiles;
    }
    if (s > smax) s = smax;
    while (s > 1 && (long long)s * tiles > kMaxItems) --s;
    return s < 1 ? 1 : s;
}

// BM x BN workgroup tile, waves arranged WM (channels) x WN (pixels).
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(NT) void gemm_gather_kernel(GemmArgs a)
{
    static_assert(WM * WN == 4, "four waves");
    constexpr int TP = BN / WN / 16; // 16-pixel MFMA tiles per wave
    constexpr int TC = BM / WM / 16; // 16-channel MFMA tiles per wave
    constexpr int PA = BN / 32;      // A rows loaded per thread and stage
    constexpr int PB = (BM + 31) / 32;
    static_assert(TP >= 1 && TC >= 1, "tile too small");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                                    // [2][BN][LDK]  gathered image-matrix slice
    float *Bs = smem + 2 * BN * LDK;                     // [2][BM][LDK]  filter-matrix slice
    int *sU = reinterpret_cast<int *>(Bs + 2 * BM * LDK); // [BN] listed pixels of this tile (-1: none)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wpx0 = (wave % WN) * (BN / WN);
    const int wch0 = (wave / WN) * (BM / WM);
    const int lrow = lane & 15; // row of the 16-row operand tiles this lane feeds
    const int lk = lane >> 4;   // k slot this lane feeds

    const int v = tid & 7;   // float4 column inside the K slice
    const int r0 = tid >> 3; // first row this thread stages

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

        // window origin of each staged row
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

        floatx4 acc[TC][TP];
#pragma unroll
        for (int j = 0; j < TC; ++j)
#pragma unroll
            for (int i = 0; i < TP; ++i) acc[j][i] = (floatx4){0.f, 0.f, 0.f, 0.f};

        float4 ra[PA], rb[PB];
        auto fetch = [&](int kc) {
            const int2 tp = a.taps[kc * (BK / 4) + v];
            const int tj = tp.y & 0xff, ti = (tp.y >> 8) & 0xff;
            const bool tv = (tp.y >> 16) != 0;
#pragma unroll
            for (int ps = 0; ps < PA; ++ps) {
                const bool ok = tv && (unsigned)(iy0[ps] + tj) < (unsigned)a.H &&
                                (unsigned)(ix0[ps] + ti) < (unsigned)a.W;
                ra[ps] = ok ? *reinterpret_cast<const float4 *>(a.x + (base[ps] + tp.x))
                            : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int ps = 0; ps < PB; ++ps)
                if (BM >= 32 || r0 + 32 * ps < BM)
                    rb[ps] = *reinterpret_cast<const float4 *>(wrow + (size_t)(32 * ps) * a.Kpad + kc * BK);
        };
        auto stage = [&](int buf) {
            float *A = As + buf * BN * LDK;
            float *B = Bs + buf * BM * LDK;
#pragma unroll
            for (int ps = 0; ps < PA; ++ps)
                *reinterpret_cast<float4 *>(A + (r0 + 32 * ps) * LDK + v * 4) = ra[ps];
#pragma unroll
            for (int ps = 0; ps < PB; ++ps)
                if (BM >= 32 || r0 + 32 * ps < BM)
                    *reinterpret_cast<float4 *>(B + (r0 + 32 * ps) * LDK + v * 4) = rb[ps];
        };

        fetch(kc0);
        stage(0);
        __syncthreads();
        for (int kc = kc0; kc < kc1; ++kc) {
            const int buf = (kc - kc0) & 1;
            if (kc + 1 < kc1) fetch(kc + 1);
            const float *A = As + buf * BN * LDK + (wpx0 + lrow) * LDK + lk * 4;
            const float *B = Bs + buf * BM * LDK + (wch0 + lrow) * LDK + lk * 4;
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                // Each lane reads four consecutive k of its row; MFMA step s then contracts
                // k = kk*16 + 4*slot + s for slot = 0..3 -- both operands use the same permutation.
                floatx4 af[TP], bf[TC];
#pragma unroll
                for (int i = 0; i < TP; ++i) af[i] = *reinterpret_cast<const floatx4 *>(A + i * 16 * LDK + kk * 16);
#pragma unroll
                for (int j = 0; j < TC; ++j) bf[j] = *reinterpret_cast<const floatx4 *>(B + j * 16 * LDK + kk * 16);
                // D = (filter rows) x (pixel columns): D[4*slot + r][lane%16] lands in this lane,
                // i.e. four consecutive channels of one pixel per accumulator.
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int j = 0; j < TC; ++j)
#pragma unroll
                        for (int i = 0; i < TP; ++i)
                            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[j][s], af[i][s], acc[j][i], 0, 0, 0);
            }
            if (kc + 1 < kc1) stage(buf ^ 1);
            __syncthreads();
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

static int pixel_tile(int bm) { return bm == 16 ? 256 : 128; }

size_t gemm_partial_bytes(int M)
{
    const int bm = gemm_channel_tile(M);
    return (size_t)kMaxItems * bm * pixel_tile(bm) * sizeof(float);
}

#define CBK_VARIANTS(X) X(16, 256, 1, 4) X(32, 128, 1, 4) X(64, 128, 2, 2) X(128, 128, 2, 2)

hipError_t gemm_prepare(void)
{
    hipError_t e = hipSuccess;
#define X(BM_, BN_, WM_, WN_)                                                                            \
    if (e == hipSuccess)                                                                                 \
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_gather_kernel<BM_, BN_, WM_, WN_>), \
                                hipFuncAttributeMaxDynamicSharedMemorySize, TileSmem<BM_, BN_>::bytes);
    CBK_VARIANTS(X)
#undef X
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
    // has work only while the tile count is below the splitting limit (384 tiles)
    long long work = (long long)384 * BN * (a.Ms / 4);
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
    case 32: return launch<32, 128, 1, 4>(st, a);
    case 64: return launch<64, 128, 2, 2>(st, a);
    default: return launch<128, 128, 2, 2>(st, a);
    }
}

hipError_t output_update(hipStream_t st, const GemmArgs &a)
{
    const int bm = gemm_channel_tile(a.M);
    switch (bm) {
    case 16: return launch_update<16, 256>(st, a);
    case 32: return launch_update<32, 128>(st, a);
    case 64: return launch_update<64, 128>(st, a);
    default: return launch_update<128, 128>(st, a);
    }
}

} // namespace cbk
