// bf16 x bf16 -> fp32 GEMM on gfx950 MFMA (v_mfma_f32_32x32x16_bf16), LDS-staged tiles.
//
//   C[M,N] = A[M,K] * W[N,K]^T        A: activations (row-major, K contiguous)
//                                      W: weights in [out, in] order (row-major, K contiguous)
//
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of one row) is
// one 16-byte read.  A workgroup owns a BM x BN output tile and one K slice; the K loop moves
// 64-wide slabs HBM -> registers -> LDS (double buffered, one barrier per slab) while the
// previous slab feeds the matrix cores.
//
// Two tile shapes:
//   cfg 0  128x128, 4 waves of 64x64   - weight streaming for M <= 128 (bandwidth-bound):
//                                         many K slices so that >= 2 workgroups per CU keep
//                                         loads in flight;
//   cfg 1  256x256, 4 waves of 128x128 - compute-bound shapes: 16 MFMAs per 8 LDS fragment
//                                         reads, all 256 accumulator registers in use.
// Workgroup ids are remapped so that each of the 8 XCDs (workgroups are dealt to them round-
// robin) gets a contiguous range of tiles, walked M-fastest in groups of 8 row tiles: the
// workgroups sharing a weight panel sit on one XCD and hit its L2.
#include "laps_internal.h"

namespace {

constexpr int BK = 64;          // k elements per slab: 128 bytes per tile row
constexpr int CHUNKS = BK / 8;  // 16-byte chunks per tile row
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;

// Tile rows are 128 bytes; chunk c of row r is stored at chunk position c ^ f(r).  f makes any 8
// consecutive rows hit 8 different 16-byte columns and any 16 consecutive rows hit 16 different
// 16-byte columns of a 256-byte bank line, for both fragment reads (lanes = consecutive rows, same
// chunk) and slab writes (8 lanes = one row, all chunks).
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row & 7) ^ ((row >> 3) & 1)); }

template <int BM, int BN, int WM, int WN>
struct Traits {
    static constexpr int NT = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static constexpr int A_LOADS = BM * CHUNKS / NT, B_LOADS = BN * CHUNKS / NT;
    static constexpr int LDS_BYTES = 2 * (BM + BN) * BK * 2;
    static_assert(BM * CHUNKS % NT == 0 && BN * CHUNKS % NT == 0, "tile rows must divide over threads");
};

struct TileCoord {
    int tm, tn, ks;
};

__device__ __forceinline__ TileCoord map_block(int bid, int tiles_m, int tiles_n, int split) {
    const int total = tiles_m * tiles_n * split;
    const int xcd = bid % NUM_XCD, idx = bid / NUM_XCD;
    const int q = total / NUM_XCD, r = total % NUM_XCD;
    const int lin = xcd * q + (xcd < r ? xcd : r) + idx;  // contiguous range per XCD
    const int per_split = tiles_m * tiles_n;
    TileCoord c;
    c.ks = lin / per_split;
    const int t = lin - c.ks * per_split;
    const int gsize = GROUP_M * tiles_n;
    const int grp = t / gsize;
    const int first_m = grp * GROUP_M;
    const int gm = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    const int in = t - grp * gsize;
    c.tm = first_m + in % gm;
    c.tn = in / gm;
    return c;
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void gemm_partial_kernel(const bf16_t* __restrict__ A,
                                                                   const bf16_t* __restrict__ W,
                                                                   float* __restrict__ P, int M, int N, int K,
                                                                   int split, int kps, int tiles_m, int tiles_n) {
    using T = Traits<BM, BN, WM, WN>;
    extern __shared__ __align__(16) unsigned char smem[];
    u32x4* As = reinterpret_cast<u32x4*>(smem);     // [2][BM][CHUNKS]
    u32x4* Bs = As + 2 * BM * CHUNKS;               // [2][BN][CHUNKS]

    const TileCoord tc = map_block(blockIdx.x, tiles_m, tiles_n, split);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const int kbeg = tc.ks * kps;
    const int kend = (kbeg + kps < K) ? (kbeg + kps) : K;
    const int KT = (kend - kbeg) / BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lk = lane >> 5;

    // slab copy assignment: 16-byte chunk c = tid + i*NT -> (row, kc)
    const u32x4* ag[T::A_LOADS];
    const u32x4* bg[T::B_LOADS];
    int a_dst[T::A_LOADS], b_dst[T::B_LOADS];
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
        const int c = tid + i * T::NT, row = c / CHUNKS, kc = c % CHUNKS;
        const int gr = (m0 + row < M) ? (m0 + row) : (M - 1);  // clamp: rows past M are never stored
        ag[i] = reinterpret_cast<const u32x4*>(A + (size_t)gr * K + kbeg) + kc;
        a_dst[i] = row * CHUNKS + swz(row, kc);
    }
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i) {
        const int c = tid + i * T::NT, row = c / CHUNKS, kc = c % CHUNKS;
        bg[i] = reinterpret_cast<const u32x4*>(W + (size_t)(n0 + row) * K + kbeg) + kc;
        b_dst[i] = row * CHUNKS + swz(row, kc);
    }

    f32x16 acc[T::MI][T::NI];
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    u32x4 ra[T::A_LOADS], rb[T::B_LOADS];
    if (KT > 0) {
#pragma unroll
        for (int i = 0; i < T::A_LOADS; ++i) ra[i] = ag[i][0];
#pragma unroll
        for (int i = 0; i < T::B_LOADS; ++i) rb[i] = bg[i][0];
#pragma unroll
        for (int i = 0; i < T::A_LOADS; ++i) As[a_dst[i]] = ra[i];
#pragma unroll
        for (int i = 0; i < T::B_LOADS; ++i) Bs[b_dst[i]] = rb[i];
    }
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = (kt + 1 < KT);
        if (more) {
#pragma unroll
            for (int i = 0; i < T::A_LOADS; ++i) ra[i] = ag[i][(kt + 1) * CHUNKS];
#pragma unroll
            for (int i = 0; i < T::B_LOADS; ++i) rb[i] = bg[i][(kt + 1) * CHUNKS];
        }
        const u32x4* as = As + cur * BM * CHUNKS;
        const u32x4* bs = Bs + cur * BN * CHUNKS;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[T::MI], bfr[T::NI];
#pragma unroll
            for (int mi = 0; mi < T::MI; ++mi) {
                const int row = wm * T::WTM + mi * 32 + lrow;
                af[mi] = __builtin_bit_cast(bf16x8, as[row * CHUNKS + swz(row, kk * 2 + lk)]);
            }
#pragma unroll
            for (int ni = 0; ni < T::NI; ++ni) {
                const int row = wn * T::WTN + ni * 32 + lrow;
                bfr[ni] = __builtin_bit_cast(bf16x8, bs[row * CHUNKS + swz(row, kk * 2 + lk)]);
            }
#pragma unroll
            for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < T::NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }
        if (more) {
            u32x4* ad = As + (cur ^ 1) * BM * CHUNKS;
            u32x4* bd = Bs + (cur ^ 1) * BN * CHUNKS;
#pragma unroll
            for (int i = 0; i < T::A_LOADS; ++i) ad[a_dst[i]] = ra[i];
#pragma unroll
            for (int i = 0; i < T::B_LOADS; ++i) bd[b_dst[i]] = rb[i];
        }
        __syncthreads();
    }

    // accumulator layout of the 32x32 MFMA: lane -> column (lane & 31); register r -> row
    // 8*(r/4) + 4*(lane/32) + r%4
    float* out = P + (size_t)tc.ks * M * N;
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < T::NI; ++ni) {
            const int n = n0 + wn * T::WTN + ni * 32 + lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * T::WTM + mi * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (m < M) out[(size_t)m * N + n] = acc[mi][ni][r];
            }
        }
}

template <int BM, int BN, int WM, int WN>
int launch_cfg(const GemmPlan& p, const bf16_t* a, const bf16_t* w, float* partial, int m, int n, int k,
               hipStream_t s) {
    using T = Traits<BM, BN, WM, WN>;
    auto kern = gemm_partial_kernel<BM, BN, WM, WN>;
    static bool attr_set = false;  // per instantiation; idempotent, so a race only repeats the call
    if (!attr_set) {
        LAPS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES));
        attr_set = true;
    }
    const int tiles_m = (m + BM - 1) / BM, tiles_n = n / BN;
    const int grid = tiles_m * tiles_n * p.split;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(T::NT), T::LDS_BYTES, s, a, w, partial, m, n, k, p.split,
                       p.k_per_split, tiles_m, tiles_n);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

}  // namespace

GemmPlan laps_gemm_plan(int m, int n, int k, int force_split) {
    GemmPlan p;
    p.cfg = (m > 128 && n % 256 == 0) ? 1 : 0;
    const int bm = p.cfg ? 256 : 128, bn = bm;
    const int tiles = ((m + bm - 1) / bm) * (n / bn);
    const int ksteps = k / BK;
    int split = 1;
    if (force_split > 0) {
        split = force_split;
    } else if (p.cfg == 0) {
        // bandwidth-bound: at least two workgroups per CU, each with >= 8 slabs of K
        split = (512 + tiles - 1) / tiles;
        const int cap = ksteps / 8 > 1 ? ksteps / 8 : 1;
        if (split > cap) split = cap;
    } else {
        // compute-bound: smallest split whose last wave of workgroups is not mostly idle
        double best = -1.0;
        for (int s = 1; s <= 8; ++s) {
            if (s > 1 && ksteps / s < 16) break;
            const int wgs = tiles * s;
            const int waves = (wgs + 255) / 256;
            const double eff = (double)wgs / (waves * 256.0);
            if (eff > best + 0.04) {
                best = eff;
                split = s;
            }
        }
    }
    if (split > ksteps) split = ksteps;
    if (split < 1) split = 1;
    const int per = (ksteps + split - 1) / split;
    p.k_per_split = per * BK;
    p.split = (ksteps + per - 1) / per;
    return p;
}

size_t laps_gemm_partial_bytes(int m, int n, int k) {
    const GemmPlan p = laps_gemm_plan(m, n, k, 0);
    return (size_t)p.split * m * n * sizeof(float);
}

int laps_gemm_launch(const GemmPlan& p, const bf16_t* a, const bf16_t* w, float* partial, int m, int n, int k,
                     hipStream_t s) {
    if (m < 1 || n < 128 || k < BK || k % BK != 0 || n % 128 != 0) {
        laps_set_error("gemm: unsupported shape m=%d n=%d k=%d (need k %% 64 == 0, n %% 128 == 0)", m, n, k);
        return LAPS_EINVAL;
    }
    if (p.cfg == 1) {
        if (n % 256 != 0) {
            laps_set_error("gemm: 256-wide tile needs n %% 256 == 0 (n=%d)", n);
            return LAPS_EINVAL;
        }
        return launch_cfg<256, 256, 2, 2>(p, a, w, partial, m, n, k, s);
    }
    return launch_cfg<128, 128, 2, 2>(p, a, w, partial, m, n, k, s);
}
