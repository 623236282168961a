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
// Two loops share these pieces.  Workgroups of 4 waves (short prompts, split key ranges) take a tile at a time:
// scores, softmax, second product, one barrier.  Workgroups of 8 waves (long prompts) run a three-stage software
// pipeline over 32-key half tiles, in which the matrix cores work on the half tiles before and after the one whose
// softmax the vector ALU is computing; its row sums also come from the matrix cores.  In both, the value the
// exponentials subtract follows the row maximum lazily, so that O is rescaled rarely.
//
// Few query rows over a long cached prefix (a short re-prefill turn) would leave most of the chip idle:
// one request of 16 new tokens is a single row block per kv head.  For such launches the key range is
// split over gridDim.z workgroups (at least 4 key tiles each); every split writes its un-normalised
// accumulator with its running maximum and row sum, and a second kernel merges the splits in a fixed
// order, so the result does not depend on scheduling.  The split count is a function of launch shapes
// only (row blocks, kv heads, page-table width), which keeps captured graphs replayable; how many of
// the splits a given sequence really uses is decided on the device from its length.
#include "laps_internal.h"

#include <type_traits>

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

    // ---- tile copy assignment: chunk c = tid + i*NTHR of the tile's 4 pages.  All chunks a wave copies in one
    // pass lie in one page, so the page id is a wave-uniform (scalar) load.
    u32x4 kreg[NLD], vreg[NLD];   // landing registers of the tile copy
    auto page_id = [&](int j0, int i) -> int {
        int pidx = j0 / LAPS_PAGE + __builtin_amdgcn_readfirstlane((tid + i * NTHR) / CPP);
        pidx = pidx < n_pages_seq ? pidx : n_pages_seq - 1;  // past the end: any valid page, masked later
        return pt[pidx];
    };
    auto chunk_offset = [&](int pg, int i) -> size_t {
        const int within = (tid + i * NTHR) % CPP;
        // an unset (-1) entry or an id outside the pool must not turn into a wild address
        const size_t page = (size_t)((pg > 0 && pg < n_pool_pages) ? pg : 0);
        return (page * n_kv + kvh) * CPP + within;
    };
    auto store_k = [&](int buf) {   // K page is [16 keys][HD]
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * NTHR;
            const int pi = c / CPP, within = c % CPP;
            const int key = pi * LAPS_PAGE + within / CPR, kc = within % CPR;
            Ks[buf][key * CPR + (CPR == 16 ? swz16(key, kc) : swz8(key, kc))] = kreg[i];
        }
    };
    auto store_v = [&](int j0, int buf) {   // V page is [HD][16 keys]: chunk = 8 consecutive keys of one head_dim index
        const bool tail = (j0 + KT > kv_len);
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = tid + i * NTHR;
            const int pi = c / CPP, within = c % CPP;
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
    };

    // MFMA row rho = lm of the first product holds key 16(a/2) + 8h + 4(a%2) + b with rho = 8a + 4h + b
    const int ra = lm >> 3, rh = (lm >> 2) & 1, rb = lm & 3;
    const int krow = 16 * (ra >> 1) + 8 * rh + 4 * (ra & 1) + rb;

    // operand fragments: K for matrix instruction g = 2 kk + sub of the first product, V^T for g = NI u2 + ni of
    // the second
    auto k_frag = [&](int kb, int g) -> bf16x8 {
        const int row = (g & 1) * 32 + krow, ch = (g >> 1) * 2 + lh;
        return __builtin_bit_cast(bf16x8, Ks[kb][row * CPR + (CPR == 16 ? swz16(row, ch) : swz8(row, ch))]);
    };
    auto v_frag = [&](int vb, int g) -> bf16x8 {
        const int row = (g % NI) * 32 + lm;
        return __builtin_bit_cast(bf16x8, Vs[vb][row * 8 + swz8(row, (g / NI) * 2 + lh)]);
    };
    // S^T = K Q^T for the 64 keys of the tile in Ks[kb] (two 32-key sub-tiles)
    auto qk_tile = [&](int kb, f32x16 (&s)[2]) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[sub][i] = 0.f;
#pragma unroll
        for (int g = 0; g < 2 * KSTEPS; ++g)
            s[g & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(kb, g), qf[g >> 1], s[g & 1], 0, 0, 0);
    };
    // causal mask, needed on diagonal tiles only (wave-uniform test by the caller)
    auto mask_tile = [&](int j0, f32x16 (&s)[2]) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int a = i >> 2, b = i & 3;
                const int key = j0 + sub * 32 + 16 * (a >> 1) + 8 * lh + 4 * (a & 1) + b;
                s[sub][i] = (key <= limit) ? s[sub][i] : -INFINITY;
            }
    };
    // online softmax of one tile's scores, one query row per lane (shared with lane^32): probabilities as the
    // second product's operand, the tile's row maximum and row sum; softmax_finish folds them into the running
    // state and rescales O when some row's maximum moved
    // The reference value m_run that the exponentials subtract follows the row maximum lazily: it moves (and O and
    // the row sum are rescaled) only when some row's maximum has grown by more than RESCALE_SLACK in log2 units, so
    // probabilities stay below 2^RESCALE_SLACK and the 64-register rescale of O is rare.  The quotient O / l does
    // not depend on the reference.
    constexpr float RESCALE_SLACK = 8.f;
    const int partner_addr = (lane ^ 32) << 2;   // ds_bpermute address of the lane that shares this lane's row
    auto from_partner = [&](float x) {
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(partner_addr, __builtin_bit_cast(int, x)));
    };
    float m_new, psum;
    bool moved;   // wave-uniform: the reference moves to m_new after this tile
    auto pick_reference = [&](float mx) -> float {   // returns what this tile's exponentials subtract
        m_new = fmaxf(m_run, mx * scale_log2e);
        moved = __builtin_amdgcn_ballot_w64(m_new > m_run + RESCALE_SLACK) != 0;
        const float m_use = moved ? m_new : m_run;
        // un-split: finite from the first tile on (key 0 is visible to every row).  A later split can start
        // on a diagonal tile in which a row sees nothing yet: keep exp2(-inf - -inf) out of the arithmetic.
        return (SPLIT && m_use == -INFINITY) ? 0.f : m_use;
    };
    auto softmax_tile = [&](f32x16 (&s)[2], bf16x8 (&pf)[2][2]) {
        float mx = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[sub][i]);
        mx = fmaxf(mx, from_partner(mx));
        const float m_sub = pick_reference(mx);
        psum = 0.f;
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
    };
    auto softmax_finish = [&]() {
        if (moved) {
            const float alpha = (SPLIT && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= alpha;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[ni][i] *= alpha;
            m_run = m_new;
        }
        l_run += psum;
    };
    // O^T += V^T P^T with the tile in Vs[vb]
    auto pv_tile = [&](int vb, bf16x8 (&pf)[2][2]) {
#pragma unroll
        for (int g = 0; g < 4 * NI; ++g)
            o[g % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag(vb, g), pf[g / (2 * NI)][(g / NI) & 1], o[g % NI], 0, 0, 0);
    };

    const auto exists = [&](int j) { return j < kv_end; };
    if constexpr (NW == 8) {
        // Long prompts.  The loop is software-pipelined three deep over 32-key half tiles: in step w the matrix
        // cores form the scores of half tile w + 1 and add half tile w - 1 to O while the vector ALU turns the scores
        // of half tile w into probabilities - one matrix instruction, one LDS fragment read and a share of the
        // softmax per slot, so both pipes are busy in every wave whatever phase the other wave of its SIMD is in.
        // Tile t occupies Ks[t&1] and Vs[t&1].  Tile step t runs the half steps 2t and 2t + 1:
        //   2t    : scores of (t, keys 32..63), softmax of (t, keys 0..31), O += (t-1, keys 32..63)
        //   barrier: K(t) and V(t-1) are done with; K(t+2) and V(t+1) leave the registers for their buffers
        //   2t + 1: scores of (t+1, keys 0..31), softmax of (t, keys 32..63), O += (t, keys 0..31)
        // and there is one tile step more than tiles (its first half adds the last half tile to O).
        // page ids (scalars) are fetched one tile step before the loads that use them
        int idk[NLD], idv[NLD];
        auto fetch_ids = [&](int jk, int jv) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) idk[i] = page_id(jk, i), idv[i] = page_id(jv, i);
        };
        auto load_k = [&]() {
#pragma unroll
            for (int i = 0; i < NLD; ++i) kreg[i] = reinterpret_cast<const u32x4*>(k_pool)[chunk_offset(idk[i], i)];
        };
        auto load_v = [&]() {
#pragma unroll
            for (int i = 0; i < NLD; ++i) vreg[i] = reinterpret_cast<const u32x4*>(v_pool)[chunk_offset(idv[i], i)];
        };
        // wave-uniform: half tile (tile at key j, half h) exists and some row of this wave sees one of its keys
        const auto visible = [&](int j, int h) { return j >= kv_begin && j < kv_end && j + 32 * h <= vis_max; };
        constexpr int NQ = KSTEPS;       // matrix instructions of each product per half tile (equal: HD / 16)
        constexpr int NS = 2 * NQ;       // slots per half step
        constexpr int MAXS = NS >= 16 ? NS / 8 : 1;   // slots that take the row maximum
        constexpr int EXP0 = MAXS + 2;   // first slot of the exponentials
        constexpr int NE = NS + 2 - EXP0;   // slots that share the 16 exponentials
        static_assert(2 * NI == NQ, "both products issue HD / 16 matrix instructions per half tile");
        // the three stages one after the other, for the first and last half steps of a wave
        auto qk_half = [&](int kb, int h, f32x16& sc) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk)
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(kb, 2 * kk + h), qf[kk], sc, 0, 0, 0);
        };
        auto mask_half = [&](int j0, int h, f32x16& sc) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int a = i >> 2, b = i & 3;
                const int key = j0 + h * 32 + 16 * (a >> 1) + 8 * lh + 4 * (a & 1) + b;
                sc[i] = (key <= limit) ? sc[i] : -INFINITY;
            }
        };
        // Row sums come from the matrix cores as well: a fragment of ones times P^T gives, in every register of the
        // result, the sum over the fragment's keys of the probabilities as the second product sees them (rounded to
        // bf16), complete in both lanes of a row.  It is added to l_run where the same probabilities are added to O.
        bf16x8 ones;
#pragma unroll
        for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
        auto softmax_half = [&](f32x16& sc, bf16x8 (&pf)[2]) {
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sc[i]);
            mx = fmaxf(mx, from_partner(mx));
            const float m_sub = pick_reference(mx);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                bf16x8 pk;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    pk[e] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sc[8 * u + e], scale_log2e, -m_sub));
                pf[u] = pk;
            }
        };
        auto pv_half = [&](int vb, int h, bf16x8 (&pf)[2]) {
#pragma unroll
            for (int g = 0; g < 2 * NI; ++g)
                o[g % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_frag(vb, (2 * h + g / NI) * NI + g % NI), pf[g / NI],
                                                                    o[g % NI], 0, 0, 0);
            f32x16 ls;
#pragma unroll
            for (int i = 0; i < 16; ++i) ls[i] = 0.f;
            ls = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf[0], ls, 0, 0, 0);
            ls = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf[1], ls, 0, 0, 0);
            l_run += ls[0];
        };
        // moves the reference to m_new after the matrix work of a half step (the probabilities just formed already
        // use it; O and l_run, which hold the half tiles before, follow here)
        auto move_reference = [&]() {
            if (moved) {
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run *= alpha;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[ni][i] *= alpha;
                m_run = m_new;
            }
        };
        // one half step.  (kb, hq): buffer and half of the scores to form into s_nxt; s_cur -> pf_cur; (vb, hv):
        // buffer and half of the V tile that goes with pf_prev
        auto half_step = [&](bool do_qk, bool do_sm, bool do_pv, int kb, int hq, f32x16& s_nxt, f32x16& s_cur,
                             bf16x8 (&pf_cur)[2], int vb, int hv, bf16x8 (&pf_prev)[2]) __attribute__((always_inline)) {
            if (do_qk && do_sm && do_pv) {
                // slot g < NS: even = first product's instruction g / 2, odd = second product's; the last two slots
                // take the row sums.  The LDS fragment of slot g + 2 is read in slot g.
                bf16x8 fr[NS + 2];
                fr[0] = k_frag(kb, hq);
                fr[1] = v_frag(vb, 2 * hv * NI);
                f32x16 ls;
#pragma unroll
                for (int i = 0; i < 16; ++i) s_nxt[i] = 0.f, ls[i] = 0.f;
                float cmax[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                float mx = 0.f, mx_other = 0.f, m_sub = 0.f;
                bf16x8 pk;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int g = 0; g < NS + 2; ++g) {
                    const int q = g >> 1;   // index within its product
                    if (g >= NS)
                        ls = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf_prev[g - NS], ls, 0, 0, 0);
                    else if (g & 1)
                        o[q % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g], pf_prev[q / NI], o[q % NI], 0, 0, 0);
                    else
                        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g], qf[q], s_nxt, 0, 0, 0);
                    if (g + 2 < NS) {
                        const int q2 = (g + 2) >> 1;
                        fr[g + 2] = ((g + 2) & 1) ? v_frag(vb, (2 * hv + q2 / NI) * NI + q2 % NI) : k_frag(kb, 2 * q2 + hq);
                    }
                    // ---- this slot's share of the softmax
                    if (g < MAXS) {   // four independent chains over 16 / MAXS values per slot
                        constexpr int PER = 16 / MAXS;
#pragma unroll
                        for (int k = 0; k < PER; ++k) cmax[k & 3] = fmaxf(cmax[k & 3], s_cur[g * PER + k]);
                    } else if (g == MAXS) {
                        mx = fmaxf(fmaxf(cmax[0], cmax[1]), fmaxf(cmax[2], cmax[3]));
                        mx_other = from_partner(mx);
                    } else if (g == MAXS + 1) {
                        m_sub = pick_reference(fmaxf(mx, mx_other));
                    } else {
#pragma unroll
                        for (int k = 0; k < 16; ++k) {
                            if ((k * NE) / 16 != g - EXP0) continue;
                            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[k], scale_log2e, -m_sub));
                            asm volatile("" : "+v"(p));   // keeps the exponential in its slot (it would sink below
                                                          // the rescale branch, out from under the matrix work)
                            pk[k & 7] = (__bf16)p;
                            if ((k & 7) == 7) pf_cur[k >> 3] = pk;
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                l_run += ls[0];
                move_reference();
            } else {
                if (do_qk) qk_half(kb, hq, s_nxt);
                if (do_sm) softmax_half(s_cur, pf_cur);
                if (do_pv) pv_half(vb, hv, pf_prev);
                if (do_sm) move_reference();
            }
        };
        f32x16 s_lo, s_hi;            // scores of keys 0..31 / 32..63 of a tile
        bf16x8 p_lo[2], p_hi[2];      // their probabilities
        auto tile_step = [&](int j0, auto parity) __attribute__((always_inline)) {
            constexpr int b = decltype(parity)::value;   // j0's tile sits in buffers b, its neighbours in b ^ 1
            {
                const bool sm = visible(j0, 0);
                if (sm && j0 + 31 > vis_min) mask_half(j0, 0, s_lo);
                half_step(visible(j0, 1), sm, visible(j0 - KT, 1), b, 1, s_hi, s_lo, p_lo, b ^ 1, 1, p_hi);
            }
            __syncthreads();
            if (exists(j0 + 2 * KT)) store_k(b);
            if (exists(j0 + KT)) store_v(j0 + KT, b ^ 1);
            if (exists(j0 + 3 * KT)) load_k();
            if (exists(j0 + 2 * KT)) load_v();
            fetch_ids(j0 + 4 * KT, j0 + 3 * KT);   // clamped to the sequence's pages: harmless past the end
            {
                const bool sm = visible(j0, 1);
                if (sm && j0 + 63 > vis_min) mask_half(j0, 1, s_hi);
                half_step(visible(j0 + KT, 0), sm, visible(j0, 0), b ^ 1, 0, s_lo, s_hi, p_hi, b, 0, p_lo);
            }
        };
        // SPLIT is never combined with this variant: a wave's first half tile always shows key 0 to every row, so
        // the running maximum is finite from the first softmax on
        static_assert(!SPLIT, "the pipelined loop serves un-split launches only");
        fetch_ids(kv_begin, kv_begin);
        load_k();
        load_v();
        fetch_ids(kv_begin + KT, kv_begin + KT);
        store_k(0);
        store_v(kv_begin, 0);
        if (exists(kv_begin + KT)) load_k();
        fetch_ids(kv_begin + 2 * KT, kv_begin + KT);
        __syncthreads();
        if (visible(kv_begin, 0)) qk_half(0, 0, s_lo);
        if (exists(kv_begin + KT)) store_k(1);
        if (exists(kv_begin + 2 * KT)) load_k();
        if (exists(kv_begin + KT)) load_v();
        fetch_ids(kv_begin + 3 * KT, kv_begin + 2 * KT);
        for (int j0 = kv_begin; j0 < kv_end + KT; j0 += 2 * KT) {   // two tile steps: the buffers swap roles
            tile_step(j0, std::integral_constant<int, 0>{});
            if (j0 + KT < kv_end + KT) tile_step(j0 + KT, std::integral_constant<int, 1>{});
        }
    } else {
        // Short prompts and key-range splits: a few tiles per workgroup, latency matters more than overlap.  The
        // page ids of a tile are fetched one step before its data, so that the two dependent loads (table entry,
        // then the page itself) do not add up on the critical path of every tile.
        int pgn[NLD];
        auto load_pages = [&](int j0) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) pgn[i] = page_id(j0, i);
        };
        auto load_tile = [&]() {   // uses the ids load_pages fetched
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const size_t off = chunk_offset(pgn[i], i);
                kreg[i] = reinterpret_cast<const u32x4*>(k_pool)[off];
                vreg[i] = reinterpret_cast<const u32x4*>(v_pool)[off];
            }
        };
        load_pages(kv_begin);
        load_tile();
        load_pages(kv_begin + KT);        // indices are clamped to the sequence's pages: harmless past the end
        store_k(0);
        store_v(kv_begin, 0);
        if (exists(kv_begin + KT)) {
            load_tile();
            load_pages(kv_begin + 2 * KT);
        }
        __syncthreads();
        int buf = 0;
        for (int j0 = kv_begin; j0 < kv_end; j0 += KT, buf ^= 1) {
            // stage the next tile (already in registers) into the other buffer, refill the registers
            if (exists(j0 + KT)) {
                store_k(buf ^ 1);
                store_v(j0 + KT, buf ^ 1);
                if (exists(j0 + 2 * KT)) {
                    load_tile();
                    load_pages(j0 + 3 * KT);
                }
            }
            if (j0 <= vis_max) {  // wave-uniform: something of this tile is visible to this wave
                f32x16 sc[2];
                bf16x8 pf[2][2];
                qk_tile(buf, sc);
                if (j0 + KT - 1 > vis_min) mask_tile(j0, sc);
                softmax_tile(sc, pf);
                softmax_finish();
                pv_tile(buf, pf);
            }
            __syncthreads();
        }
    }

    // ---- normalise and store: lane owns row r; register i of sub-tile ni is head_dim index
    //      ni*32 + 8*(i/4) + 4*(lane/32) + i%4
    // the pipelined loop holds complete row sums, the plain one a lane's share
    const float l_tot = (NW == 8) ? l_run : l_run + __shfl_xor(l_run, 32, 64);
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
