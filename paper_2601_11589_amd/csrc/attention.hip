// Ragged, paged, causal grouped-query flash attention for gfx950.
//
// One workgroup = one (sequence, kv head, block of query rows).  A "query row" is a (new token t,
// query head g of the kv head's group) pair, numbered r = t*G + g, so the G query heads that share a
// kv head are packed into the MFMA row dimension and every K/V page is fetched once for all of them.
// The workgroup walks the sequence's pages (cached prefix first, then the new tokens, which the QKV
// step has already appended) in tiles of 64 keys: coalesced 4 KB page reads -> registers -> LDS.
//
// Both products are issued transposed so that a lane owns one query row end to end:
//   S^T = K Q^T   (A = K fragment from LDS, B = Q fragment held in registers)
//   O^T = V^T P^T (A = V^T fragment from LDS - V pages are stored [head_dim][16 tokens], B = P)
// With the 32x32 accumulator layout (lane -> column, registers -> rows) the softmax statistics of a
// row live in one lane and its partner lane^32: row max and row sum need a single cross-lane
// exchange, and the O rescale is a per-lane scalar.  K rows are read from LDS through the
// permutation key(8a + 4h + b) = 16(a/2) + 8h + 4(a%2) + b, which makes the eight probabilities a
// lane holds in accumulator registers 8u..8u+7 exactly the eight consecutive keys its P fragment
// must supply to the second product - no shuffles between the two MFMA stages.
#include "laps_internal.h"

namespace {

constexpr int KT = 64;      // keys per tile (4 pages)

__device__ __forceinline__ int swz8(int row, int c) { return c ^ ((row & 7) ^ ((row >> 3) & 1)); }
__device__ __forceinline__ int swz16(int row, int c) { return c ^ (row & 15); }

// per-sequence number of query-row blocks and their exclusive prefix sum (single workgroup)
__global__ __launch_bounds__(256) void attn_sched_kernel(const int* __restrict__ new_len, int n_seq, int group,
                                                          int rows_per_wg, int* __restrict__ tile_start) {
    __shared__ int buf[256];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n_seq; base += 256) {
        const int i = base + threadIdx.x;
        const int v = (i < n_seq) ? (new_len[i] * group + rows_per_wg - 1) / rows_per_wg : 0;
        buf[threadIdx.x] = v;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {  // inclusive Hillis-Steele scan
            const int add = (threadIdx.x >= o) ? buf[threadIdx.x - o] : 0;
            __syncthreads();
            buf[threadIdx.x] += add;
            __syncthreads();
        }
        const int c = carry;
        if (i < n_seq) tile_start[i] = c + buf[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 255) carry = c + buf[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) tile_start[n_seq] = carry;
}

// NW waves per workgroup, one 32-row query tile per wave: rows per workgroup = 32 * NW.  With NW = 8
// two waves share a SIMD, so one wave's softmax (VALU, exp) overlaps the other's MFMAs.
template <int HD, int NW>
__global__ __launch_bounds__(NW * 64) void attn_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ out,
                                                        const bf16_t* __restrict__ k_pool,
                                                        const bf16_t* __restrict__ v_pool,
                                                        const int* __restrict__ row_start,
                                                        const int* __restrict__ new_len,
                                                        const int* __restrict__ prefix_len,
                                                        const int* __restrict__ page_table, int max_pages,
                                                        const int* __restrict__ tile_start, int n_seq, int n_q,
                                                        int n_kv, float scale_log2e) {
    constexpr int NTHR = NW * 64;
    constexpr int CPR = HD / 8;            // 16-byte chunks per K row
    constexpr int CPP = HD * 2;            // 16-byte chunks per page (K and V alike)
    constexpr int NLD = KT * CPR / NTHR;   // chunk loads per thread per tile, K and V each
    constexpr int KSTEPS = HD / 16;        // MFMA k-steps over head_dim
    constexpr int NI = HD / 32;            // output sub-tiles over head_dim
    constexpr int ROWS = 32 * NW;
    static_assert(KT * CPR % NTHR == 0, "tile chunks must divide over the threads");

    __shared__ __align__(16) u32x4 Ks[2][KT * CPR];   // double buffered: one barrier per tile
    __shared__ __align__(16) u32x4 Vs[2][HD * 8];

    const int item = blockIdx.x;
    if (item >= tile_start[n_seq]) return;
    int lo = 0, hi = n_seq;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tile_start[mid] <= item) lo = mid; else hi = mid;
    }
    const int seq = lo;
    const int qtile = item - tile_start[seq];
    const int kvh = blockIdx.y;
    const int G = n_q / n_kv;
    const int L = new_len[seq], H = prefix_len[seq];
    const int n_rows = L * G;
    const int kv_len = H + L;
    const int n_pages_seq = (kv_len + LAPS_PAGE - 1) / LAPS_PAGE;
    const int R0 = qtile * ROWS;
    if (R0 >= n_rows) return;
    const int last_row_wg = (R0 + ROWS < n_rows ? R0 + ROWS : n_rows) - 1;
    const int kv_end = H + last_row_wg / G + 1;  // keys visible to the last row of this block
    const int* pt = page_table + (size_t)seq * max_pages;
    const size_t tok0 = (size_t)row_start[seq];
    const int q_stride = n_q * HD;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 31, lh = lane >> 5;

    // ---- this wave's 32 query rows: Q fragments stay in registers for the whole kernel
    const int base = R0 + wave * 32;
    const int row_id = base + lm;
    const int rc = row_id < n_rows ? row_id : n_rows - 1;
    const int tq = rc / G, gq = rc - tq * G;
    const int limit = H + tq;                                        // last visible key of this lane's row
    const int vis_min = H + (base < n_rows ? base : n_rows - 1) / G;  // wave-uniform: every row sees keys <= vis_min
    const int vis_max = (base < n_rows) ? H + (base + 31 < n_rows ? base + 31 : n_rows - 1) / G : -1;
    bf16x8 qf[KSTEPS];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(q + (tok0 + tq) * q_stride + (size_t)(kvh * G + gq) * HD);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, qp[kk * 2 + lh]);
    }
    f32x16 o[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[ni][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;   // running max (in log2 units, already scaled) and partial row sum

    // ---- tile copy assignment: chunk c = tid + i*NTHR of the tile's 4 pages
    u32x4 kreg[NLD], vreg[NLD];
    auto load_tile = [&](int j0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * NTHR;
            const int pi = c / CPP, within = c % CPP;
            int pidx = j0 / LAPS_PAGE + pi;
            pidx = pidx < n_pages_seq ? pidx : n_pages_seq - 1;  // past the end: any valid page, masked later
            const int pg = pt[pidx];
            const size_t page = (size_t)(pg > 0 ? pg : 0);  // an unset (-1) entry must not turn into a wild address
            const size_t off = ((page * n_kv + kvh) * CPP + within);
            kreg[i] = reinterpret_cast<const u32x4*>(k_pool)[off];
            vreg[i] = reinterpret_cast<const u32x4*>(v_pool)[off];
        }
    };
    auto store_tile = [&](int j0, int buf) {
        const bool tail = (j0 + KT > kv_len);
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * NTHR;
            const int pi = c / CPP, within = c % CPP;
            {   // K page is [16 keys][HD]
                const int key = pi * LAPS_PAGE + within / CPR, kc = within % CPR;
                Ks[buf][key * CPR + (CPR == 16 ? swz16(key, kc) : swz8(key, kc))] = kreg[i];
            }
            {   // V page is [HD][16 keys]: chunk = 8 consecutive keys of one head_dim index
                const int e = within / 2, half = within & 1;
                u32x4 v = vreg[i];
                if (tail) {  // zero keys >= kv_len so that 0 * garbage cannot produce NaN
                    const int nvalid = kv_len - (j0 + pi * LAPS_PAGE + half * 8);
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        unsigned x = v[w];
                        if (2 * w + 1 >= nvalid) x &= 0x0000ffffu;
                        if (2 * w >= nvalid) x = 0u;
                        v[w] = x;
                    }
                }
                Vs[buf][e * 8 + swz8(e, pi * 2 + half)] = v;
            }
        }
    };

    // MFMA row rho = lm of the first product holds key 16(a/2) + 8h + 4(a%2) + b with rho = 8a + 4h + b
    const int ra = lm >> 3, rh = (lm >> 2) & 1, rb = lm & 3;
    const int krow = 16 * (ra >> 1) + 8 * rh + 4 * (ra & 1) + rb;

    load_tile(0);
    store_tile(0, 0);
    if (KT < kv_end) load_tile(KT);
    __syncthreads();
    int buf = 0;
    for (int j0 = 0; j0 < kv_end; j0 += KT, buf ^= 1) {
        // stage the next tile (already in registers) into the other buffer, refill the registers
        if (j0 + KT < kv_end) {
            store_tile(j0 + KT, buf ^ 1);
            if (j0 + 2 * KT < kv_end) load_tile(j0 + 2 * KT);
        }
        if (j0 <= vis_max) {  // wave-uniform: something of this tile is visible to this wave
            // ---- S^T = K Q^T for the 64 keys of the tile (two 32-key sub-tiles)
            f32x16 s[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[sub][i] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    const int row = sub * 32 + krow;
                    const int ch = kk * 2 + lh;
                    const bf16x8 kf = __builtin_bit_cast(
                        bf16x8, Ks[buf][row * CPR + (CPR == 16 ? swz16(row, ch) : swz8(row, ch))]);
                    s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[sub], 0, 0, 0);
                }
            }
            // ---- causal mask (diagonal tiles only) + online softmax, one query row per lane (shared with lane^32)
            if (j0 + KT - 1 > vis_min) {
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int a = i >> 2, b = i & 3;
                        const int key = j0 + sub * 32 + 16 * (a >> 1) + 8 * lh + 4 * (a & 1) + b;
                        s[sub][i] = (key <= limit) ? s[sub][i] : -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[sub][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx * scale_log2e);  // finite from the first tile on (key 0 is visible)
            bf16x8 pf[2][2];
            float psum = 0.f;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    bf16x8 pk;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[sub][8 * u + e], scale_log2e, -m_new));
                        psum += p;
                        pk[e] = (__bf16)p;
                    }
                    pf[sub][u] = pk;
                }
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {  // some row's maximum moved: rescale
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run *= alpha;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[ni][i] *= alpha;
                m_run = m_new;
            }
            l_run += psum;
            // ---- O^T += V^T P^T
#pragma unroll
            for (int u2 = 0; u2 < 4; ++u2) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const int row = ni * 32 + lm;
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, Vs[buf][row * 8 + swz8(row, u2 * 2 + lh)]);
                    o[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u2 >> 1][u2 & 1], o[ni], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }

    // ---- normalise and store: lane owns row r; register i of sub-tile ni is head_dim index
    //      ni*32 + 8*(i/4) + 4*(lane/32) + i%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (row_id < n_rows) {
        const float inv = 1.f / l_tot;
        bf16_t* op = out + (tok0 + tq) * q_stride + (size_t)(kvh * G + gq) * HD;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                u32x2 w;
                w.x = pack_bf16x2(o[ni][4 * a] * inv, o[ni][4 * a + 1] * inv);
                w.y = pack_bf16x2(o[ni][4 * a + 2] * inv, o[ni][4 * a + 3] * inv);
                *reinterpret_cast<u32x2*>(op + ni * 32 + 8 * a + 4 * lh) = w;
            }
    }
}

template <int HD, int NW>
int launch_attn(const bf16_t* q, bf16_t* out, const bf16_t* k_pool, const bf16_t* v_pool, const int* row_start,
                const int* new_len, const int* prefix_len, const int* page_table, int max_pages, const int* tile_start,
                int n_seq, int max_items, int n_q, int n_kv, hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
    hipLaunchKernelGGL((attn_kernel<HD, NW>), dim3(max_items, n_kv), dim3(NW * 64), 0, s, q, out, k_pool, v_pool,
                       row_start, new_len, prefix_len, page_table, max_pages, tile_start, n_seq, n_q, n_kv, scale_log2e);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

}  // namespace

// Query-row blocking for a batch: rows per workgroup (128 or 256) and an upper bound on the number
// of (sequence, row block) work items.  Depends only on shapes known to the host.
static void attn_blocking(int n_seq, int n_tokens, int group, int* mt, int* max_items) {
    const long total_rows = (long)n_tokens * group;
    *mt = (total_rows > 128L * n_seq) ? 2 : 1;  // average rows per sequence above one 128-row block
    const int rows_per_wg = 128 * *mt;
    // every sequence contributes ceil(rows/rows_per_wg) blocks: at most rows/rows_per_wg + 1
    *max_items = (int)(total_rows / rows_per_wg) + n_seq;
}

// Work-item table for laps_launch_attention; depends on the batch only, so a layer stack builds it once.
int laps_launch_attn_sched(const int* new_len, int n_seq, int n_tokens, int* tile_start, int n_q, int n_kv,
                           hipStream_t s) {
    int mt, max_items;
    attn_blocking(n_seq, n_tokens, n_q / n_kv, &mt, &max_items);
    hipLaunchKernelGGL(attn_sched_kernel, dim3(1), dim3(256), 0, s, new_len, n_seq, n_q / n_kv, 128 * mt, tile_start);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_attention(const bf16_t* q, bf16_t* out, const bf16_t* k_pool, const bf16_t* v_pool,
                          const int* row_start, const int* new_len, const int* prefix_len, const int* page_table,
                          int max_pages, int n_seq, int n_tokens, const int* tile_start, int n_q, int n_kv, int hd,
                          hipStream_t s) {
    int mt, max_items;
    attn_blocking(n_seq, n_tokens, n_q / n_kv, &mt, &max_items);
    if (hd == 128) {
        if (mt == 2) return launch_attn<128, 8>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, n_seq, max_items, n_q, n_kv, s);
        return launch_attn<128, 4>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, n_seq, max_items, n_q, n_kv, s);
    }
    if (hd == 64) {
        if (mt == 2) return launch_attn<64, 8>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, n_seq, max_items, n_q, n_kv, s);
        return launch_attn<64, 4>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, n_seq, max_items, n_q, n_kv, s);
    }
    laps_set_error("attention: head_dim %d not supported (64 or 128)", hd);
    return LAPS_EINVAL;
}
