// bf16 x bf16 -> fp32 GEMM on gfx950 MFMA (v_mfma_f32_32x32x16_bf16), LDS-staged tiles.
//
//   C[M,N] = A[M,K] * W[N,K]^T        A: activations (row-major, K contiguous)
//                                      W: weights in [out, in] order (row-major, K contiguous)
//
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of one row) is one
// 16-byte read.  A workgroup owns a BM x BN output tile and one K slice.  The K loop moves 64-wide
// slabs HBM -> registers -> LDS (two LDS buffers) and is software-pipelined by hand:
//   * fragments of k-step kk+1 are read from LDS into a second register set before the MFMAs of
//     k-step kk are issued, so LDS latency hides behind 8..16 MFMAs;
//   * the registers holding slab kt+1 are written to the other LDS buffer in the middle of slab kt
//     and immediately reloaded with slab kt+2 from HBM (about 1.75 slabs of prefetch distance);
//   * the one barrier per slab sits in the middle of the last k-step's MFMAs and waits on LDS
//     traffic only, never on the HBM loads in flight.
// Epilogues: raw K-slice partial sums (split-K, reduced deterministically by the row kernels in
// elementwise.hip), residual add (fp32 out), or SwiGLU on interleaved gate/up columns (bf16 out).
//
// Workgroup ids are remapped so that each of the 8 XCDs (workgroups are dealt to them round-robin)
// gets a contiguous range of tiles, walked M-fastest in groups of 8 row tiles: the workgroups
// sharing a weight panel sit on one XCD and hit its L2.
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

// LDS-only barrier: waits for this wave's LDS reads/writes, not for global loads in flight.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int BM, int BN, int WM, int WN>
struct Traits {
    static constexpr int NT = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static constexpr int A_LOADS = BM * CHUNKS / NT, B_LOADS = BN * CHUNKS / NT;
    static constexpr int LDS_BYTES = 2 * (BM + BN) * BK * 2;
    static_assert(BM * CHUNKS % NT == 0 && BN * CHUNKS % NT == 0, "tile rows must divide over threads");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
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

struct GemmArgs {
    const bf16_t* A;
    const bf16_t* W;
    int M, N, K, split, kps, tiles_m, tiles_n;
    float* out_f32;        // EPI_PARTIAL: [split][M][N]; EPI_RESID: [M][N]
    const float* resid;    // EPI_RESID: [M][N] (may alias out_f32)
    bf16_t* out_bf16;      // EPI_SWIGLU: [M][N/2]
    const int* row_live;   // [M] or NULL: rows with a negative entry are padding - skinny tiles skip their A loads,
                           // every tile shape skips a row tile that holds nothing else (its output is then not written)
};

// Writes a workgroup's accumulators with the requested epilogue.  Accumulator layout of the 32x32 MFMA:
// lane -> column (lane & 31); register r -> row 8*(r/4) + 4*(lane/32) + r%4.
template <typename T, int EPI>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[T::MI][T::NI], const GemmArgs& g, int ks, int m0, int n0,
                                           int wm, int wn, int lrow, int lk) {
    const int M = g.M, N = g.N;
    if constexpr (EPI == EPI_PARTIAL || EPI == EPI_RESID) {
        float* out = g.out_f32 + (EPI == EPI_PARTIAL ? (size_t)ks * M * N : (size_t)0);
#pragma unroll
        for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < T::NI; ++ni) {
                const int n = n0 + wn * T::WTN + ni * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * T::WTM + mi * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                    if (m < M) {
                        const size_t o = (size_t)m * N + n;
                        out[o] = (EPI == EPI_RESID) ? g.resid[o] + acc[mi][ni][r] : acc[mi][ni][r];
                    }
                }
            }
    } else {  // EPI_SWIGLU: sub-tile 2j holds gate columns, sub-tile 2j+1 the matching up columns
        static_assert(EPI != EPI_SWIGLU || T::NI % 2 == 0, "SwiGLU epilogue pairs 32-column sub-tiles");
        const int half_n = N / 2;
#pragma unroll
        for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
            for (int j = 0; j < T::NI / 2; ++j) {
                const int col = (n0 + wn * T::WTN) / 2 + j * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * T::WTM + mi * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                    if (m < M) {
                        const float gt = acc[mi][2 * j][r], up = acc[mi][2 * j + 1][r];
                        g.out_bf16[(size_t)m * half_n + col] = f32_to_bf16(gt / (1.f + __expf(-gt)) * up);
                    }
                }
            }
    }
}

// WS = number of register sets that stage slabs: WS slabs (A and W chunks alike - loads return in
// issue order, so a shallower A stream would throttle the W stream) are in flight per workgroup.
// WS > 1 is for the bandwidth-bound skinny shapes; the K loop is then unrolled WS times so every set
// index is static, and the K slice must hold a multiple of WS slabs.
template <int BM, int BN, int WM, int WN, int EPI, int WS>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(const GemmArgs g) {
    using T = Traits<BM, BN, WM, WN>;
    extern __shared__ __align__(16) unsigned char smem[];
    u32x4* As = reinterpret_cast<u32x4*>(smem);  // [2][BM][CHUNKS]
    u32x4* Bs = As + 2 * BM * CHUNKS;            // [2][BN][CHUNKS]

    const int M = g.M, N = g.N, K = g.K;
    const TileCoord tc = map_block(blockIdx.x, g.tiles_m, g.tiles_n, g.split);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;
    const int kbeg = tc.ks * g.kps;
    const int kend = (kbeg + g.kps < K) ? (kbeg + g.kps) : K;
    const int KT = (kend - kbeg) / BK;

    constexpr bool NT = (BM <= 128);  // skinny tiles only
    const int tid = threadIdx.x;
    if (g.row_live != nullptr) {  // a row tile made of padding only has nothing to compute (and nothing reads its output)
        bool any = false;
        for (int r = tid; r < BM; r += T::NT) any |= (m0 + r < M) && g.row_live[m0 + r] >= 0;
        if (!__syncthreads_or(any)) return;
    }
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lk = lane >> 5;

    // slab copy assignment: 16-byte chunk c = tid + i*NT -> (row, kc)
    const u32x4* ag[T::A_LOADS];
    const u32x4* bg[T::B_LOADS];
    int a_dst[T::A_LOADS], b_dst[T::B_LOADS];
    // Skinny tiles: a CU keeps a bounded number of requests in flight, and the A slab's share of them
    // (a third with 256 columns) is taken from the weight stream; rows past M and padding rows are
    // therefore not loaded at all - their staging registers stay zero.
    bool a_live[T::A_LOADS];
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
        const int c = tid + i * T::NT, row = c / CHUNKS, kc = c % CHUNKS;
        const int gr = (m0 + row < M) ? (m0 + row) : (M - 1);  // clamp: rows past M are never stored
        ag[i] = reinterpret_cast<const u32x4*>(g.A + (size_t)gr * K + kbeg) + kc;
        a_dst[i] = row * CHUNKS + swz(row, kc);
        a_live[i] = !NT || (m0 + row < M && (g.row_live == nullptr || g.row_live[gr] >= 0));
    }
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i) {
        const int c = tid + i * T::NT, row = c / CHUNKS, kc = c % CHUNKS;
        bg[i] = reinterpret_cast<const u32x4*>(g.W + (size_t)(n0 + row) * K + kbeg) + kc;
        b_dst[i] = row * CHUNKS + swz(row, kc);
    }
    // fragment read offsets (in 16-byte chunks) inside one LDS buffer, per k-step
    int a_src[T::MI], b_src[T::NI];
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi) a_src[mi] = (wm * T::WTM + mi * 32 + lrow) * CHUNKS;
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni) b_src[ni] = (wn * T::WTN + ni * 32 + lrow) * CHUNKS;
    const int a_sw = (lrow & 7) ^ ((lrow >> 3) & 1);  // rows differ by multiples of 32: same swizzle key

    f32x16 acc[T::MI][T::NI];
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    u32x4 rra[WS][T::A_LOADS];   // staged A slabs: slab j lives in set j % WS
    if constexpr (NT) {
#pragma unroll
        for (int w = 0; w < WS; ++w)
#pragma unroll
            for (int i = 0; i < T::A_LOADS; ++i) rra[w][i] = u32x4{0u, 0u, 0u, 0u};
    }
    u32x4 rrb[WS][T::B_LOADS];   // staged W slabs, same rule
    bf16x8 fa[2][T::MI], fb[2][T::NI];
    constexpr int NM = T::MI * T::NI;            // MFMAs per k-step
    constexpr int NF = T::MI + T::NI;            // fragment reads per k-step
    constexpr int NC = T::A_LOADS + T::B_LOADS;  // slab copy operations (global load + LDS store pairs)
    constexpr int NC0 = (NC + 1) / 2;            // copies handled in k-step 0; the rest in k-step 1

    auto clampk = [&](int kt) { return kt < KT ? kt : KT - 1; };  // tail: reload a valid slab, never used
    // copy op i of the slab pipeline: i < A_LOADS moves an A chunk, else a W chunk held in set `ws`
    auto gload_one = [&](int i, int kt, int ws) {
        if (i < T::A_LOADS) {
            if constexpr (NT) {
                if (a_live[i]) rra[ws][i] = ag[i][clampk(kt) * CHUNKS];
            } else {
                rra[ws][i] = ag[i][clampk(kt) * CHUNKS];
            }
        } else {
            // weights are read once: streaming (non-temporal) loads keep them from evicting the A slabs,
            // which every workgroup on the CU and on the XCD re-reads, out of L1 / L2
            const u32x4* src = bg[i - T::A_LOADS] + clampk(kt) * CHUNKS;
            rrb[ws][i - T::A_LOADS] = NT ? __builtin_nontemporal_load(src) : *src;
        }
    };
    auto lstore_one = [&](int i, int buf, int ws) {
        if (i < T::A_LOADS) As[buf * BM * CHUNKS + a_dst[i]] = rra[ws][i];
        else Bs[buf * BN * CHUNKS + b_dst[i - T::A_LOADS]] = rrb[ws][i - T::A_LOADS];
    };
    // order of need by the MFMA sequence (mi-major): A row block 0, every B column block, remaining A
    auto fload_one = [&](int i, int buf, int kk, int set) {
        const int ch = (kk * 2 + lk) ^ a_sw;
        if (i == 0) fa[set][0] = __builtin_bit_cast(bf16x8, As[buf * BM * CHUNKS + a_src[0] + ch]);
        else if (i <= T::NI) fb[set][i - 1] = __builtin_bit_cast(bf16x8, Bs[buf * BN * CHUNKS + b_src[i - 1] + ch]);
        else fa[set][i - T::NI] = __builtin_bit_cast(bf16x8, As[buf * BM * CHUNKS + a_src[i - T::NI] + ch]);
    };
    auto mma_one = [&](int i, int set) {
        const int mi = i / T::NI, ni = i % T::NI;
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][mi], fb[set][ni], acc[mi][ni], 0, 0, 0);
    };

    // prologue: slab 0 through the registers into LDS buffer 0, then A slab 1 and W slabs 1..WS in flight
#pragma unroll
    for (int i = 0; i < NC; ++i) gload_one(i, 0, 0);
#pragma unroll
    for (int i = 0; i < NC; ++i) lstore_one(i, 0, 0);
#pragma unroll
    for (int w = 1; w <= WS; ++w)
#pragma unroll
        for (int i = 0; i < NC; ++i) gload_one(i, w, w % WS);
    lds_barrier();
#pragma unroll
    for (int i = 0; i < NF; ++i) fload_one(i, 0, 0, 0);

    // One memory operation is slotted behind each MFMA so that the matrix pipe never waits for a
    // clump of LDS / HBM instructions to issue (one wave per SIMD: nothing else would feed it).
    //   k-step 0: MFMAs on set 0 | reads of k-step 1 fragments -> set 1 | first half of the slab copy
    //   k-step 1: MFMAs on set 1 | reads of k-step 2 fragments -> set 0 | second half of the slab copy
    //   k-step 2: MFMAs on set 0 | reads of k-step 3 fragments -> set 1
    //   k-step 3: MFMAs on set 1 | barrier half way | reads of the next slab's k-step 0 -> set 0
    // A slab copy = store the staged slab kt+1 to the other LDS buffer, then reload the set just freed
    // with slab kt+1+WS from HBM.  The tail iterations keep the same
    // instruction stream (no branches in the pipeline): they re-store and re-load the last slab, which
    // nothing reads afterwards.
    for (int kt0 = 0; kt0 < KT; kt0 += WS) {
#pragma unroll
        for (int u = 0; u < WS; ++u) {
            const int kt = kt0 + u;
            const int cur = (WS == 1) ? (kt & 1) : (u & 1);  // WS is 1 or even
            const int ws = (u + 1) % WS;                     // set holding W slab kt+1
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mma_one(i, 0);
#pragma unroll
                for (int o = i; o < NF + NC0; o += NM) {
                    if (o < NF) fload_one(o, cur, 1, 1);
                    else {
                        lstore_one(o - NF, cur ^ 1, ws);
                        gload_one(o - NF, kt + 1 + WS, ws);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mma_one(i, 1);
#pragma unroll
                for (int o = i; o < NF + (NC - NC0); o += NM) {
                    if (o < NF) fload_one(o, cur, 2, 0);
                    else {
                        lstore_one(NC0 + o - NF, cur ^ 1, ws);
                        gload_one(NC0 + o - NF, kt + 1 + WS, ws);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mma_one(i, 0);
#pragma unroll
                for (int o = i; o < NF; o += NM) fload_one(o, cur, 3, 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            constexpr int NH = NM / 2;
#pragma unroll
            for (int i = 0; i < NH; ++i) mma_one(i, 1);
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = NH; i < NM; ++i) {
                mma_one(i, 1);
#pragma unroll
                for (int o = i - NH; o < NF; o += NM - NH) fload_one(o, cur ^ 1, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    store_tile<T, EPI>(acc, g, tc.ks, m0, n0, wm, wn, lrow, lk);
}

template <int BM, int BN, int WM, int WN, int EPI, int WS = 1>
int launch_tile(const GemmArgs& a, hipStream_t s) {
    using T = Traits<BM, BN, WM, WN>;
    auto kern = gemm_kernel<BM, BN, WM, WN, EPI, WS>;
    static bool attr_set = false;  // per instantiation; idempotent, so a race only repeats the call
    if (!attr_set) {
        LAPS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     T::LDS_BYTES));
        attr_set = true;
    }
    const int grid = a.tiles_m * a.tiles_n * a.split;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(T::NT), T::LDS_BYTES, s, a);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

struct TileDef {
    int bm, bn;
    double eff;  // relative MFMA efficiency of the tile shape (operand reuse), 256x256 = 1
};
// index = GemmPlan::cfg
constexpr TileDef kTiles[] = {
    {128, 128, 0.70},  // 0: skinny fallback (n % 256 != 0), 4 waves of 64x64
    {128, 64, 0.50},   // 1: skinny fallback (n % 128 != 0)
    {256, 256, 1.00},  // 2: 4 waves of 128x128
    {256, 224, 0.93},  // 3: 4 waves of 64x224 (N = 7168 -> 32 column tiles)
    {256, 160, 0.85},  // 4: 4 waves of 64x160 (N = 5120 -> 32 column tiles)
    {128, 256, 0.80},  // 5: skinny, 8 waves of 64x64: one workgroup per CU, A slab shared by 256 columns
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

}  // namespace

void laps_gemm_tile_dims(int cfg, int* bm, int* bn) {
    *bm = (cfg >= 0 && cfg < kNumTiles) ? kTiles[cfg].bm : 0;
    *bn = (cfg >= 0 && cfg < kNumTiles) ? kTiles[cfg].bn : 0;
}

// Picks tile shape and K split.
GemmPlan laps_gemm_plan(int m, int n, int k, int force_split, int want_epi) {
    GemmPlan p;
    const int ksteps = k / BK;
    auto finish = [&](int cfg, int split) {
        if (split > ksteps) split = ksteps;
        if (split < 1) split = 1;
        int per = (ksteps + split - 1) / split;
        // skinny tiles keep 2 slabs in flight: every K slice must then hold a multiple of 2 slabs
        p.ws = 1;
        if (kTiles[cfg].bm == 128 && ksteps % 2 == 0) {
            per = (per + 1) / 2 * 2;
            p.ws = 2;
        }
        p.cfg = cfg;
        p.k_per_split = per * BK;
        p.split = (ksteps + per - 1) / per;
        p.epi = (p.split == 1) ? want_epi : EPI_PARTIAL;
        return p;
    };
    if (m <= 128) {
        // Bandwidth-bound.  A CU keeps a bounded number of requests in flight, and the A slab that every
        // workgroup re-reads per K step (L2 hits) takes its share of them from the weight stream: a
        // 256-column tile halves the A share of a 128-column one, which decides the wide projections
        // (gate/up: 5.3 against 4.4 TB/s of weights).  A narrow
        // projection (q/k/v, o: 20-28 tiles of 256 columns) never gets near that limit; it pays for the
        // K split that has to fill the chip - every slice writes m*n fp32 partial sums that a reduce
        // kernel reads back - and for the short pipeline of each slice.  128-column tiles need half the
        // split; they win where the 256-column slices would be shorter than 24 K slabs (measured with
        // cold weights at m = 128: q/k/v 33.8 -> 26.7 us, o 29.0 -> 22.4, 7B-shaped down 43.8 -> 37.4;
        // the 32B down projection, 36 slabs per slice, is even and stays on 256 columns).  At most 256
        // workgroups either way: a streaming kernel with 257 leaves one CU with twice the work.
        auto auto_split = [&](int c) {
            const int min_steps = c == 5 ? 8 : 16;   // K slabs per slice below which the pipeline is all prologue
            int sp = 256 / (n / kTiles[c].bn);
            const int cap = (ksteps + min_steps / 2) / min_steps;
            sp = sp > cap ? cap : sp;
            return sp < 1 ? 1 : sp;
        };
        int cfg;
        if (n % 256 == 0 && (n % 128 != 0 || ksteps / auto_split(5) >= 24)) cfg = 5;
        else cfg = (n % 128 == 0) ? 0 : 1;
        if (cfg == 1 && want_epi == EPI_SWIGLU) want_epi = EPI_PARTIAL;
        const int split = force_split > 0 ? force_split : auto_split(cfg);
        return finish(cfg, split);
    }
    // compute-bound: minimise rounds(tiles*split over 256 CUs) * per-workgroup MFMA time + the
    // time to write and re-read the partial sums of a split
    double best = 1e30;
    int best_cfg = 2, best_split = 1;
    for (int cfg = 2; cfg <= 4; ++cfg) {
        const TileDef& t = kTiles[cfg];
        if (n % t.bn != 0) continue;
        if (want_epi == EPI_SWIGLU && cfg != 2) continue;
        const int tiles = ((m + t.bm - 1) / t.bm) * (n / t.bn);
        for (int s = 1; s <= 8; ++s) {
            if (force_split > 0 && s != force_split) continue;
            if (s > 1 && ksteps / s < 16) break;
            const long wgs = (long)tiles * s;
            const long rounds = (wgs + 255) / 256;
            const double wg_flops = 2.0 * t.bm * t.bn * (double)k / s;
            const double t_mma = rounds * wg_flops / (2.5e15 / 256 * 0.62 * t.eff);
            const double t_part = s > 1 ? (2.0 * s * m * (double)n * 4) / 4.0e12 + 4e-6 : 0.0;
            const double cost = t_mma + t_part;
            if (cost < best) {
                best = cost;
                best_cfg = cfg;
                best_split = s;
            }
        }
    }
    if (best >= 1e30) {  // no wide tile divides n: fall back to the 128- or 64-wide panels
        const int cfg = (n % 128 == 0) ? 0 : 1;
        if (cfg == 1 && want_epi == EPI_SWIGLU) want_epi = EPI_PARTIAL;
        return finish(cfg, force_split > 0 ? force_split : 1);
    }
    return finish(best_cfg, best_split);
}

size_t laps_gemm_partial_bytes(int m, int n, int k) {
    // upper bound over the epilogue kinds the layer driver may request
    size_t b = 0;
    for (int e = 0; e < 3; ++e) {
        const GemmPlan p = laps_gemm_plan(m, n, k, 0, e);
        const size_t t = p.split > 1 ? (size_t)p.split * m * n * sizeof(float) : 0;
        b = t > b ? t : b;
    }
    // QKV always goes through the partial buffer (its epilogue is a separate kernel)
    const size_t one = (size_t)m * n * sizeof(float);
    return b > one ? b : one;
}

int laps_gemm_launch(const GemmPlan& p, const bf16_t* a, const bf16_t* w, int m, int n, int k, float* out_f32,
                     const float* resid, bf16_t* out_bf16, const int* row_live, hipStream_t s) {
    if (m < 1 || n < 64 || k < BK || k % BK != 0 || p.cfg < 0 || p.cfg >= kNumTiles || n % kTiles[p.cfg].bn != 0) {
        laps_set_error("gemm: unsupported shape m=%d n=%d k=%d for tile %d", m, n, k, p.cfg);
        return LAPS_EINVAL;
    }
    if (p.ws != 1 && (p.k_per_split / BK) % p.ws != 0) {
        laps_set_error("gemm: K slice of %d slabs is not a multiple of the %d weight stages", p.k_per_split / BK, p.ws);
        return LAPS_EINVAL;
    }
    if (p.epi != EPI_PARTIAL && p.split != 1) {
        laps_set_error("gemm: fused epilogue needs a single K slice");
        return LAPS_EINVAL;
    }
    GemmArgs g;
    g.A = a;
    g.W = w;
    g.M = m;
    g.N = n;
    g.K = k;
    g.split = p.split;
    g.kps = p.k_per_split;
    g.tiles_m = (m + kTiles[p.cfg].bm - 1) / kTiles[p.cfg].bm;
    g.tiles_n = n / kTiles[p.cfg].bn;
    g.out_f32 = out_f32;
    g.resid = resid;
    g.out_bf16 = out_bf16;
    g.row_live = row_live;
#define LAPS_TILE_CASE(cfg, BM, BN, WM, WN, EPI, WS) \
    case ((cfg) * 4 + (EPI)) * 8 + (WS): return launch_tile<BM, BN, WM, WN, EPI, WS>(g, s)
    switch ((p.cfg * 4 + p.epi) * 8 + p.ws) {
        LAPS_TILE_CASE(0, 128, 128, 2, 2, EPI_PARTIAL, 1);
        LAPS_TILE_CASE(0, 128, 128, 2, 2, EPI_PARTIAL, 2);
        LAPS_TILE_CASE(0, 128, 128, 2, 2, EPI_RESID, 1);
        LAPS_TILE_CASE(0, 128, 128, 2, 2, EPI_RESID, 2);
        LAPS_TILE_CASE(0, 128, 128, 2, 2, EPI_SWIGLU, 1);
        LAPS_TILE_CASE(0, 128, 128, 2, 2, EPI_SWIGLU, 2);
        LAPS_TILE_CASE(1, 128, 64, 2, 2, EPI_PARTIAL, 1);
        LAPS_TILE_CASE(1, 128, 64, 2, 2, EPI_PARTIAL, 2);
        LAPS_TILE_CASE(1, 128, 64, 2, 2, EPI_RESID, 1);
        LAPS_TILE_CASE(1, 128, 64, 2, 2, EPI_RESID, 2);
        LAPS_TILE_CASE(2, 256, 256, 2, 2, EPI_PARTIAL, 1);
        LAPS_TILE_CASE(2, 256, 256, 2, 2, EPI_RESID, 1);
        LAPS_TILE_CASE(2, 256, 256, 2, 2, EPI_SWIGLU, 1);
        LAPS_TILE_CASE(3, 256, 224, 4, 1, EPI_PARTIAL, 1);
        LAPS_TILE_CASE(3, 256, 224, 4, 1, EPI_RESID, 1);
        LAPS_TILE_CASE(4, 256, 160, 4, 1, EPI_PARTIAL, 1);
        LAPS_TILE_CASE(4, 256, 160, 4, 1, EPI_RESID, 1);
        LAPS_TILE_CASE(5, 128, 256, 2, 4, EPI_PARTIAL, 1);
        LAPS_TILE_CASE(5, 128, 256, 2, 4, EPI_PARTIAL, 2);
        LAPS_TILE_CASE(5, 128, 256, 2, 4, EPI_RESID, 1);
        LAPS_TILE_CASE(5, 128, 256, 2, 4, EPI_RESID, 2);
        LAPS_TILE_CASE(5, 128, 256, 2, 4, EPI_SWIGLU, 1);
        LAPS_TILE_CASE(5, 128, 256, 2, 4, EPI_SWIGLU, 2);
        default: break;
    }
#undef LAPS_TILE_CASE
    laps_set_error("gemm: no kernel for tile %d with epilogue %d", p.cfg, p.epi);
    return LAPS_EINVAL;
}
