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

template <int BM, int BN>
struct TileSmem {
    static constexpr int a_floats = BN * LDK;
    static constexpr int b_floats = BM * LDK;
    static constexpr int bytes = 2 * (a_floats + b_floats) * 4 + BN * 4;
};

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
    float *As = smem;                                    // [2][BN][LDK]
    float *Bs = smem + 2 * BN * LDK;                     // [2][BM][LDK]
    int *sU = reinterpret_cast<int *>(Bs + 2 * BM * LDK); // [BN] listed pixels of this tile (-1: none)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wpx0 = (wave % WN) * (BN / WN);
    const int wch0 = (wave / WN) * (BM / WM);
    const int lrow = lane & 15; // row of the 16x16 tile this lane feeds
    const int lk = lane >> 4;   // k slot this lane feeds

    const int v = tid & 7;   // float4 column inside the K slice
    const int r0 = tid >> 3; // first row this thread stages

    const int n = *a.count;
    const int mtiles = a.Mpad / BM;
    const int tiles = ((n + BN - 1) / BN) * mtiles;
    const int nk = a.Kpad / BK;

    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int pt = tile / mtiles;
        const int mt = tile - pt * mtiles;

        __syncthreads(); // previous tile's LDS reads are done
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

        floatx4 acc[TP][TC];
#pragma unroll
        for (int i = 0; i < TP; ++i)
#pragma unroll
            for (int j = 0; j < TC; ++j) acc[i][j] = (floatx4){0.f, 0.f, 0.f, 0.f};

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

        fetch(0);
        stage(0);
        __syncthreads();
        for (int kc = 0; kc < nk; ++kc) {
            const int buf = kc & 1;
            if (kc + 1 < nk) fetch(kc + 1);
            const float *A = As + buf * BN * LDK + (wpx0 + lrow) * LDK + lk * 4;
            const float *B = Bs + buf * BM * LDK + (wch0 + lrow) * LDK + lk * 4;
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                // Each lane reads four consecutive k of its row; MFMA step s then contracts
                // k = kk*16 + 4*slot + s for slot = 0..3 -- A and B use the same permutation.
                floatx4 af[TP], bf[TC];
#pragma unroll
                for (int i = 0; i < TP; ++i) af[i] = *reinterpret_cast<const floatx4 *>(A + i * 16 * LDK + kk * 16);
#pragma unroll
                for (int j = 0; j < TC; ++j) bf[j] = *reinterpret_cast<const floatx4 *>(B + j * 16 * LDK + kk * 16);
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int i = 0; i < TP; ++i)
#pragma unroll
                        for (int j = 0; j < TC; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i][s], bf[j][s], acc[i][j], 0, 0, 0);
            }
            if (kc + 1 < nk) stage(buf ^ 1);
            __syncthreads();
        }

        // Output update: lane holds D[4*(lane/16) + r][lane%16] of every 16x16 tile
        // (row = listed pixel, column = channel).  Bias, activation, scatter.
#pragma unroll
        for (int j = 0; j < TC; ++j) {
            const int ch = mt * BM + wch0 + j * 16 + lrow;
            const float bv = a.bias[ch];
#pragma unroll
            for (int i = 0; i < TP; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int g = sU[wpx0 + i * 16 + lk * 4 + r];
                    if (g >= 0 && ch < a.M) {
                        float val = acc[i][j][r] + bv;
                        if (a.relu) val = fmaxf(val, 0.0f);
                        a.out[(size_t)g * a.Ms + ch] = val;
                    }
                }
        }
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
    const long long maxtiles = (long long)((a.max_pixels + BN - 1) / BN) * (a.Mpad / BM);
    int grid = (int)(maxtiles < 2048 ? maxtiles : 2048);
    if (grid < 1) grid = 1;
    constexpr int smem_bytes = TileSmem<BM, BN>::bytes;
    gemm_gather_kernel<BM, BN, WM, WN><<<dim3(grid), dim3(NT), smem_bytes, st>>>(a);
    return hipGetLastError();
}

hipError_t gemm_gather(hipStream_t st, const GemmArgs &a)
{
    const int bm = gemm_channel_tile(a.M);
    if (a.Mpad % bm != 0 || a.Kpad % BK != 0 || a.Cs % 4 != 0) return hipErrorInvalidValue;
    switch (bm) {
    case 16: return launch<16, 256, 1, 4>(st, a);
    case 32: return launch<32, 128, 1, 4>(st, a);
    case 64: return launch<64, 128, 2, 2>(st, a);
    default: return launch<128, 128, 2, 2>(st, a);
    }
}

} // namespace cbk
