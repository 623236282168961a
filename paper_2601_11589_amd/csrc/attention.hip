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
//
// Few query rows over a long cached prefix (a short re-prefill turn) would leave most of the chip idle:
// one request of 16 new tokens is a single row block per kv head.  For such launches the key range is
// split over gridDim.z workgroups (at least 4 key tiles each); every split writes its un-normalised
// accumulator with its running maximum and row sum, and a second kernel merges the splits in a fixed
// order, so the result does not depend on scheduling.  The split count is a function of launch shapes
// only (row blocks, kv heads, page-table width), which keeps captured graphs replayable; how many of
// the splits a given sequence really uses is decided on the device from its length.
#include "laps_internal.h"

namespace {

constexpr int KT = 64;      // keys per tile (4 pages)

__device__ __forceinline__ int swz8(int row, int c) { return c ^ ((row & 7) ^ ((row >> 3) & 1)); }
__device__ __forceinline__ int swz16(int row, int c) { return c ^ (row & 15); }

// per-sequence number of query-row blocks, their exclusive prefix sum, and the sequence of every work item
// (single workgroup).  The item table spares each attention workgroup a chain of dependent loads.
__global__ __launch_bounds__(256) void attn_sched_kernel(const int* __restrict__ new_len, int n_seq, int group,
                                                          int rows_per_wg, int* __restrict__ tile_start,
                                                          int* __restrict__ item_seq, int max_items) {
    __shared__ int buf[256];
    __shared__ int carry;
    laps_dev_attn_sched(new_len, n_seq, group, rows_per_wg, tile_start, item_seq, max_items, buf, &carry);
}

// NW waves per workgroup, one 32-row query tile per wave: rows per workgroup = 32 * NW.  With NW = 8
// two waves share a SIMD, so one wave's softmax (VALU, exp) overlaps the other's MFMAs.
// key tiles per split (lower bound) and the split geometry shared by the attention and the merge kernel
constexpr int MIN_TILES_PER_SPLIT = 4;
__device__ __forceinline__ void split_geometry(int kv_end, int n_split, int* eff, int* per) {
    const int nt = (kv_end + KT - 1) / KT;
    int e = nt / MIN_TILES_PER_SPLIT;
    e = e < 1 ? 1 : (e > n_split ? n_split : e);
    *eff = e;
    *per = (nt + e - 1) / e;
}

// A prefix length that the page table cannot hold (a corrupted or stale array) must neither index past the
// table nor make a workgroup walk millions of key tiles: cut to what max_pages pages can address.
__device__ __forceinline__ int clamp_prefix(int h, int new_len, int max_pages) {
    const int room = max_pages * LAPS_PAGE - new_len;
    h = h < room ? h : room;
    return h > 0 ? h : 0;
}

// Two waves per SIMD in every variant (second launch-bound argument): with 4 waves per workgroup that is two
// resident workgroups per compute unit, which the key-streaming launches need to cover the memory latency.
template <int HD, int NW, bool SPLIT>
__global__ __launch_bounds__(NW * 64, 2) void attn_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ out,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml,
                                                        const bf16_t* __restrict__ k_pool,
                                                        const bf16_t* __restrict__ v_pool,
                                                        const int* __restrict__ row_start,
                                                        const int* __restrict__ new_len,
                                                        const int* __restrict__ prefix_len,
                                                        const int* __restrict__ page_table, int max_pages,
                                                        const int* __restrict__ tile_start,
                                                        const int* __restrict__ item_seq, int n_seq, int n_q,
                                                        int n_kv, float scale_log2e, int n_pool_pages, int n_tokens) {
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
    const int seq = item_seq[item];
    const int qtile = item - tile_start[seq];
    const int kvh = blockIdx.y;
    const int G = n_q / n_kv;
    const int L = new_len[seq], H = clamp_prefix(prefix_len[seq], L, max_pages);
    // row offsets come from the caller's device array: rows outside the batch are never touched, whatever it holds
    const int rs = row_start[seq];
    if (rs < 0 || L > n_tokens - rs) return;
    const int n_rows = L * G;
    const int kv_len = H + L;
    // never index past the table's width, whatever the lengths say (keys beyond it then repeat the last page)
    const int n_pages_need = (kv_len + LAPS_PAGE - 1) / LAPS_PAGE;
    const int n_pages_seq = n_pages_need < max_pages ? n_pages_need : max_pages;
    const int R0 = qtile * ROWS;
    if (R0 >= n_rows) return;
    const int last_row_wg = (R0 + ROWS < n_rows ? R0 + ROWS : n_rows) - 1;
    const int kv_end_all = H + last_row_wg / G + 1;  // keys visible to the last row of this block
    int kv_begin = 0, kv_end = kv_end_all, eff = 1;
    if (SPLIT) {
        int per;
        split_geometry(kv_end_all, (int)gridDim.z, &eff, &per);
        const int z = blockIdx.z;
        if (z >= eff || z * per * KT >= kv_end_all) return;   // this split has no keys: the merge skips it too
        kv_begin = z * per * KT;
        kv_end = (z + 1) * per * KT < kv_end_all ? (z + 1) * per * KT : kv_end_all;
    }
    const int* pt = page_table + (size_t)seq * max_pages;
    const size_t tok0 = (size_t)rs;
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
    // The page ids of a tile are fetched one step before its data, so that the two dependent loads (table entry,
    // then the page itself) do not add up on the critical path of every tile.
    u32x4 kreg[NLD], vreg[NLD];
    int pgn[NLD];
    auto load_pages = [&](int j0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            int pidx = j0 / LAPS_PAGE + (tid + i * NTHR) / CPP;
            pidx = pidx < n_pages_seq ? pidx : n_pages_seq - 1;  // past the end: any valid page, masked later
            pgn[i] = pt[pidx];
        }
    };
    auto load_tile = [&](int j0) {   // uses the ids load_pages(j0) fetched
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * NTHR;
            const int within = c % CPP;
            const int pg = pgn[i];
            // an unset (-1) entry or an id outside the pool must not turn into a wild address
            const size_t page = (size_t)((pg > 0 && pg < n_pool_pages) ? pg : 0);
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

    auto compute_tile = [&](int j0, int buf) {
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
            // un-split: finite from the first tile on (key 0 is visible to every row).  A later split can start
            // on a diagonal tile in which a row sees nothing yet: keep exp2(-inf - -inf) out of the arithmetic.
            const float m_new = fmaxf(m_run, mx * scale_log2e);
            const float m_sub = (SPLIT && m_new == -INFINITY) ? 0.f : m_new;
            bf16x8 pf[2][2];
            float psum = 0.f;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    bf16x8 pk;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[sub][8 * u + e], scale_log2e, -m_sub));
                        psum += p;
                        pk[e] = (__bf16)p;
                    }
                    pf[sub][u] = pk;
                }
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {  // some row's maximum moved: rescale
                const float alpha = (SPLIT && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
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
    };
    load_pages(kv_begin);
    load_tile(kv_begin);
    load_pages(kv_begin + KT);        // indices are clamped to the sequence's pages: harmless past the end
    store_tile(kv_begin, 0);
    if (kv_begin + KT < kv_end) {
        load_tile(kv_begin + KT);
        load_pages(kv_begin + 2 * KT);
    }
    __syncthreads();
    int buf = 0;
    for (int j0 = kv_begin; j0 < kv_end; j0 += KT, buf ^= 1) {
        // stage the next tile (already in registers) into the other buffer, refill the registers.  (A second
        // register set, two tiles in flight, spills at head_dim 128: the landing registers are the limit.)
        if (j0 + KT < kv_end) {
            store_tile(j0 + KT, buf ^ 1);
            if (j0 + 2 * KT < kv_end) {
                load_tile(j0 + 2 * KT);
                load_pages(j0 + 3 * KT);
            }
        }
        compute_tile(j0, buf);
        __syncthreads();
    }

    // ---- normalise and store: lane owns row r; register i of sub-tile ni is head_dim index
    //      ni*32 + 8*(i/4) + 4*(lane/32) + i%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (SPLIT && eff > 1) {
        // partial result of this key range: accumulator as [4-float chunk][row] so that the 32 rows of a half
        // wave write consecutive 16-byte pieces; (running max, row sum) per row
        if (row_id < n_rows) {
            const size_t blk = ((size_t)item * n_kv + kvh) * gridDim.z + blockIdx.z;
            const int row = wave * 32 + lm;
            f32x4* po = reinterpret_cast<f32x4*>(part_o) + blk * (size_t)(HD / 4) * ROWS;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 w;
                    w.x = o[ni][4 * a]; w.y = o[ni][4 * a + 1]; w.z = o[ni][4 * a + 2]; w.w = o[ni][4 * a + 3];
                    po[(size_t)(ni * 8 + 2 * a + lh) * ROWS + row] = w;
                }
            if (lh == 0) {
                float* pm = part_ml + blk * (size_t)(2 * ROWS);
                pm[row] = m_run;
                pm[ROWS + row] = l_tot;
            }
        }
        return;
    }
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

// Merges the key-range splits of attn_kernel<.., SPLIT = true> in a fixed order: out = sum_z 2^(m_z - M) O_z /
// sum_z 2^(m_z - M) l_z with M = max_z m_z.  A workgroup covers the 128 rows of one work item and one 4-float
// slice of head_dim; its four groups of 128 threads take the splits z = g, g + 4, g + 8, ... (more loads in flight than one
// thread per row could issue) and their four partial sums are added in the order g = 0, 1, 2, 3.
constexpr int MERGE_GROUPS = 4;
template <int HD>
__global__ __launch_bounds__(128 * MERGE_GROUPS) void attn_merge_kernel(
    bf16_t* __restrict__ out, const float* __restrict__ part_o, const float* __restrict__ part_ml,
    const int* __restrict__ row_start, const int* __restrict__ new_len, const int* __restrict__ prefix_len,
    const int* __restrict__ tile_start, const int* __restrict__ item_seq, int n_seq, int n_q, int n_kv, int n_split,
    int max_pages, int n_tokens) {
    constexpr int ROWS = 128;
    __shared__ float red_m[MERGE_GROUPS][ROWS];
    __shared__ float red_l[MERGE_GROUPS][ROWS];
    __shared__ f32x4 red_o[MERGE_GROUPS][ROWS];
    const int item = blockIdx.x;
    if (item >= tile_start[n_seq]) return;
    const int seq = item_seq[item], qtile = item - tile_start[seq], kvh = blockIdx.y;
    const int G = n_q / n_kv;
    const int L = new_len[seq], H = clamp_prefix(prefix_len[seq], L, max_pages);   // as in attn_kernel
    const int rs = row_start[seq];
    if (rs < 0 || L > n_tokens - rs) return;                                          // as in attn_kernel
    const int n_rows = L * G, R0 = qtile * ROWS;
    if (R0 >= n_rows) return;
    const int last_row_wg = (R0 + ROWS < n_rows ? R0 + ROWS : n_rows) - 1;
    const int kv_end_all = H + last_row_wg / G + 1;
    int eff, per;
    split_geometry(kv_end_all, n_split, &eff, &per);
    if (eff == 1) return;   // the attention kernel wrote the final rows itself (uniform over the workgroup)
    const int nt = (kv_end_all + KT - 1) / KT;
    const int used = (nt + per - 1) / per < eff ? (nt + per - 1) / per : eff;   // splits that had keys
    const int row = threadIdx.x % ROWS, g = threadIdx.x / ROWS, row_id = R0 + row;
    const bool live = row_id < n_rows;
    const size_t blk0 = ((size_t)item * n_kv + kvh) * n_split;
    const float* pm = part_ml + blk0 * (size_t)(2 * ROWS) + row;
    // every load below is independent of the others: unrolled so that many are in flight at once
    float m_g = -INFINITY;
    if (live) {
#pragma unroll 4
        for (int z = g; z < used; z += MERGE_GROUPS) m_g = fmaxf(m_g, pm[(size_t)z * 2 * ROWS]);
    }
    red_m[g][row] = m_g;
    __syncthreads();
    float m_all = red_m[0][row];
#pragma unroll
    for (int k = 1; k < MERGE_GROUPS; ++k) m_all = fmaxf(m_all, red_m[k][row]);
    const int c = blockIdx.z;   // one 4-float chunk of head_dim per workgroup
    const f32x4* po = reinterpret_cast<const f32x4*>(part_o) + (blk0 * (size_t)(HD / 4) + c) * ROWS + row;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float l_g = 0.f;
    if (live) {
#pragma unroll 4
        for (int z = g; z < used; z += MERGE_GROUPS) {
            const float w = __builtin_amdgcn_exp2f(pm[(size_t)z * 2 * ROWS] - m_all);
            const f32x4 v = po[(size_t)z * (HD / 4) * ROWS];
            l_g = __builtin_fmaf(w, pm[(size_t)z * 2 * ROWS + ROWS], l_g);
            acc.x = __builtin_fmaf(w, v.x, acc.x);
            acc.y = __builtin_fmaf(w, v.y, acc.y);
            acc.z = __builtin_fmaf(w, v.z, acc.z);
            acc.w = __builtin_fmaf(w, v.w, acc.w);
        }
    }
    red_l[g][row] = l_g;
    red_o[g][row] = acc;
    __syncthreads();
    if (g != 0 || !live) return;
    float l_all = red_l[0][row];
    f32x4 o4 = red_o[0][row];
#pragma unroll
    for (int k = 1; k < MERGE_GROUPS; ++k) {
        l_all += red_l[k][row];
        const f32x4 t = red_o[k][row];
        o4.x += t.x; o4.y += t.y; o4.z += t.z; o4.w += t.w;
    }
    const float inv = 1.f / l_all;
    const int tq = row_id / G, gq = row_id - tq * G;
    bf16_t* op = out + ((size_t)rs + tq) * (size_t)(n_q * HD) + (size_t)(kvh * G + gq) * HD;
    u32x2 o2;
    o2.x = pack_bf16x2(o4.x * inv, o4.y * inv);
    o2.y = pack_bf16x2(o4.z * inv, o4.w * inv);
    *reinterpret_cast<u32x2*>(op + 4 * c) = o2;
}

template <int HD, int NW>
int launch_attn(const bf16_t* q, bf16_t* out, const bf16_t* k_pool, const bf16_t* v_pool, const int* row_start,
                const int* new_len, const int* prefix_len, const int* page_table, int max_pages, const int* tile_start,
                const int* item_seq, int n_seq, int max_items, int n_q, int n_kv, int n_pool_pages, int n_tokens,
                hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
    hipLaunchKernelGGL((attn_kernel<HD, NW, false>), dim3(max_items, n_kv), dim3(NW * 64), 0, s, q, out, nullptr, nullptr,
                       k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq,
                       n_q, n_kv, scale_log2e, n_pool_pages, n_tokens);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

template <int HD>
int launch_attn_split(const bf16_t* q, bf16_t* out, float* part, const bf16_t* k_pool, const bf16_t* v_pool,
                      const int* row_start, const int* new_len, const int* prefix_len, const int* page_table,
                      int max_pages, const int* tile_start, const int* item_seq, int n_seq, int max_items, int n_split,
                      int n_q, int n_kv, int n_pool_pages, int n_tokens, hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
    const size_t blocks = (size_t)max_items * n_kv * n_split;
    float* part_o = part;
    float* part_ml = part + blocks * 128 * HD;
    hipLaunchKernelGGL((attn_kernel<HD, 4, true>), dim3(max_items, n_kv, n_split), dim3(256), 0, s, q, out, part_o, part_ml,
                       k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq,
                       n_q, n_kv, scale_log2e, n_pool_pages, n_tokens);
    LAPS_LAUNCH_CHECK();
    hipLaunchKernelGGL((attn_merge_kernel<HD>), dim3(max_items, n_kv, HD / 4), dim3(128 * MERGE_GROUPS), 0, s, out, part_o, part_ml,
                       row_start, new_len, prefix_len, tile_start, item_seq, n_seq, n_q, n_kv, n_split, max_pages, n_tokens);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

}  // namespace

// Upper bound on the workgroups of a key-split launch, and the bytes of partial results it needs.
static constexpr int kSplitTargetBlocks = 512;   // aim for two workgroups per compute unit
static constexpr int kSplitBelowBlocks = 256;    // launches with fewer un-split workgroups than this are split
static constexpr int kSplitMax = 64;

size_t laps_attn_partial_bytes(int hd, int max_pages) {
    // page tables too narrow for two splits never take the split path (same test as attn_blocking)
    if (((long)max_pages * LAPS_PAGE + KT - 1) / KT < 2 * MIN_TILES_PER_SPLIT) return 0;
    // blocks0 < kSplitBelowBlocks and n_split <= ceil(kSplitTargetBlocks / blocks0) give fewer than
    // kSplitTargetBlocks + kSplitBelowBlocks workgroups, each with 128 rows of (hd + 2) floats
    return (size_t)(kSplitTargetBlocks + kSplitBelowBlocks) * 128 * (size_t)(hd + 2) * sizeof(float);
}

// Query-row blocking for a batch: rows per workgroup (128 or 256), an upper bound on the number of
// (sequence, row block) work items, and the number of key-range splits.  Depends only on shapes known to
// the host (a captured graph must replay with the same grid whatever the lengths staged into it).
static void attn_blocking(int n_seq, int n_tokens, int group, int n_kv, int max_pages, int* mt, int* max_items,
                          int* n_split) {
    const long total_rows = (long)n_tokens * group;
    const long items1 = total_rows / 128 + n_seq;      // bound with 128-row blocks
    const int max_kv_tiles = (max_pages * LAPS_PAGE + KT - 1) / KT;
    *n_split = 1;
    if (items1 * n_kv < kSplitBelowBlocks && max_kv_tiles >= 2 * MIN_TILES_PER_SPLIT) {
        const int blocks0 = (int)items1 * n_kv;
        int ns = (kSplitTargetBlocks + blocks0 - 1) / blocks0;
        ns = ns < max_kv_tiles / MIN_TILES_PER_SPLIT ? ns : max_kv_tiles / MIN_TILES_PER_SPLIT;
        ns = ns < kSplitMax ? ns : kSplitMax;
        if (ns > 1) {
            *n_split = ns;
            *mt = 1;
            *max_items = (int)items1;
            return;
        }
    }
    *mt = (total_rows > 128L * n_seq) ? 2 : 1;  // average rows per sequence above one 128-row block
    const int rows_per_wg = 128 * *mt;
    // every sequence contributes ceil(rows/rows_per_wg) blocks: at most rows/rows_per_wg + 1
    *max_items = (int)(total_rows / rows_per_wg) + n_seq;
}

void laps_attn_plan(int n_seq, int n_tokens, int group, int n_kv, int max_pages, int* rows_per_wg, int* max_items,
                    int* n_split, int* min_tiles_per_split) {
    int mt = 1;
    attn_blocking(n_seq, n_tokens, group, n_kv, max_pages, &mt, max_items, n_split);
    *rows_per_wg = 128 * mt;
    *min_tiles_per_split = MIN_TILES_PER_SPLIT;
}

// Work-item table for laps_launch_attention; depends on the batch only, so a layer stack builds it once.
size_t laps_attn_item_table_bytes(int max_tokens, int max_seqs, int group) {
    return ((size_t)max_tokens * group / 128 + max_seqs + 1) * sizeof(int);
}

int laps_launch_attn_sched(const int* new_len, int n_seq, int n_tokens, int max_pages, int* tile_start, int* item_seq,
                           int n_q, int n_kv, hipStream_t s) {
    int mt, max_items, n_split;
    attn_blocking(n_seq, n_tokens, n_q / n_kv, n_kv, max_pages, &mt, &max_items, &n_split);
    hipLaunchKernelGGL(attn_sched_kernel, dim3(1), dim3(256), 0, s, new_len, n_seq, n_q / n_kv, 128 * mt, tile_start,
                       item_seq, max_items);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_attention(const bf16_t* q, bf16_t* out, const bf16_t* k_pool, const bf16_t* v_pool,
                          const int* row_start, const int* new_len, const int* prefix_len, const int* page_table,
                          int max_pages, int n_seq, int n_tokens, const int* tile_start, const int* item_seq,
                          float* partial, int n_q, int n_kv, int hd, int n_pool_pages, hipStream_t s) {
    int mt, max_items, n_split;
    attn_blocking(n_seq, n_tokens, n_q / n_kv, n_kv, max_pages, &mt, &max_items, &n_split);
    if (n_split > 1) {
        if (!partial) {
            laps_set_error("attention: key-split launch needs the partial-result workspace");
            return LAPS_EINVAL;
        }
        if (hd == 128) return launch_attn_split<128>(q, out, partial, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq, max_items, n_split, n_q, n_kv, n_pool_pages, n_tokens, s);
        if (hd == 64) return launch_attn_split<64>(q, out, partial, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq, max_items, n_split, n_q, n_kv, n_pool_pages, n_tokens, s);
    }
    if (hd == 128) {
        if (mt == 2) return launch_attn<128, 8>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq, max_items, n_q, n_kv, n_pool_pages, n_tokens, s);
        return launch_attn<128, 4>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq, max_items, n_q, n_kv, n_pool_pages, n_tokens, s);
    }
    if (hd == 64) {
        if (mt == 2) return launch_attn<64, 8>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq, max_items, n_q, n_kv, n_pool_pages, n_tokens, s);
        return launch_attn<64, 4>(q, out, k_pool, v_pool, row_start, new_len, prefix_len, page_table, max_pages, tile_start, item_seq, n_seq, max_items, n_q, n_kv, n_pool_pages, n_tokens, s);
    }
    laps_set_error("attention: head_dim %d not supported (64 or 128)", hd);
    return LAPS_EINVAL;
}
