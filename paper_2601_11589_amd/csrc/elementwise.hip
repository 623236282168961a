// Row-wise kernels around the GEMMs: token metadata, RMSNorm, split-K reductions fused with the
// layer's element-wise steps (residual + next RMSNorm, RoPE + KV append, SwiGLU), weight packing
// and KV cache moves.  All are bandwidth-trivial next to the GEMMs; they use one workgroup per
// row with 16-byte accesses.
#include "laps_internal.h"

namespace {

constexpr int ROW_THREADS = 256;

__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();  // red may still be read from a previous call
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < ROW_THREADS / 64; ++w) t += red[w];
    return t;
}

// ------------------------------------------------------------------ rope table (fp64 evaluation)
__global__ void rope_table_kernel(float2* table, int max_pos, int half, double theta, int hd) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= max_pos * half) return;
    const int p = i / half, j = i % half;
    const double inv_freq = pow(theta, -2.0 * (double)j / (double)hd);
    const double ang = (double)p * inv_freq;
    table[i] = make_float2((float)cos(ang), (float)sin(ang));
}

// ------------------------------------------------------------------ token metadata
// Owning sequence of a row by binary search over row_start, then absolute position and KV slot
// (page * 16 + offset) of the token; -1 for padding rows.
__device__ __forceinline__ void token_meta(int row, int n_seq, const int* __restrict__ row_start,
                                           const int* __restrict__ seq_len, const int* __restrict__ prefix_len,
                                           const int* __restrict__ page_table, int max_pages, int n_pool_pages, int* pos_out,
                                           int* slot_out) {
    int lo = 0, hi = n_seq;  // find s with row_start[s] <= row < row_start[s+1]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (row_start[mid] <= row) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int t = row - row_start[s];
    const int cap = row_start[s + 1] - row_start[s];
    int l = seq_len ? seq_len[s] : cap;
    l = l > cap ? cap : l;
    int pos = -1, slot = -1;
    if (t >= 0 && t < l) {
        const int h = prefix_len[s];
        pos = (h > 0 ? h : 0) + t;
        // a position past the table's width, an unset (-1) entry or a page id outside the pool: no cache write
        const int pi = pos / LAPS_PAGE;
        const int page = pi < max_pages ? page_table[(size_t)s * max_pages + pi] : -1;
        slot = (page >= 0 && page < n_pool_pages) ? page * LAPS_PAGE + pos % LAPS_PAGE : -1;
    }
    *pos_out = pos;
    *slot_out = slot;
}

// One thread per row (and per sequence for the clamped lengths).
__global__ void prep_kernel(int n_rows, int n_seq, const int* __restrict__ row_start, const int* __restrict__ seq_len,
                            const int* __restrict__ prefix_len, const int* __restrict__ page_table, int max_pages,
                            int n_pool_pages, int* __restrict__ new_len_out, int* __restrict__ tok_pos,
                            int* __restrict__ tok_slot) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row < n_seq) {
        const int cap = row_start[row + 1] - row_start[row];
        int l = seq_len ? seq_len[row] : cap;
        l = l > cap ? cap : l;
        new_len_out[row] = l < 0 ? 0 : l;
    }
    if (row >= n_rows) return;
    int pos, slot;
    token_meta(row, n_seq, row_start, seq_len, prefix_len, page_table, max_pages, n_pool_pages, &pos, &slot);
    tok_pos[row] = pos;
    tok_slot[row] = slot;
}

// ------------------------------------------------------------------ RMSNorm: fp32 row -> bf16 row
// One row with ROW_THREADS threads; xr may be any fp32 row of d values, red holds ROW_THREADS / 64 floats of LDS.
__device__ __forceinline__ void rmsnorm_row(const f32x4* __restrict__ xr, const bf16_t* __restrict__ w,
                                            bf16_t* __restrict__ out_row, int d, float eps, float* red) {
    float ss = 0.f;
    for (int i = threadIdx.x; i < d / 4; i += ROW_THREADS) {
        const f32x4 v = xr[i];
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    const float inv = rsqrtf(block_sum(ss, red) / (float)d + eps);
    u32x2* orow = reinterpret_cast<u32x2*>(out_row);
    const u32x2* wr = reinterpret_cast<const u32x2*>(w);
    for (int i = threadIdx.x; i < d / 4; i += ROW_THREADS) {
        const f32x4 v = xr[i];
        const u32x2 g = wr[i];
        u32x2 o;
        o.x = pack_bf16x2(v.x * inv * __uint_as_float(g.x << 16), v.y * inv * __uint_as_float(g.x & 0xffff0000u));
        o.y = pack_bf16x2(v.z * inv * __uint_as_float(g.y << 16), v.w * inv * __uint_as_float(g.y & 0xffff0000u));
        orow[i] = o;
    }
}

__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_kernel(const float* __restrict__ x,
                                                               const bf16_t* __restrict__ w, bf16_t* __restrict__ out,
                                                               int d, float eps, const int* __restrict__ row_live) {
    __shared__ float red[ROW_THREADS / 64];
    const size_t row = blockIdx.x;
    if (row_live && row_live[row] < 0) return;  // padding row: nothing reads its output
    rmsnorm_row(reinterpret_cast<const f32x4*>(x + row * d), w, out + row * d, d, eps, red);
}

// ------------------------------------------------------------------ sum K slices + residual (+ RMSNorm)
// x_out[row] = resid[row] (or 0 if resid is null) + sum_s partial[s][row]; optionally
// r_out[row] = rmsnorm(x_out[row]) in bf16.  One workgroup of 512 threads per row; the row stays in
// registers between the two passes (d <= 4 * 512 * MAXV).
constexpr int RESID_THREADS = 512;

__device__ __forceinline__ float block_sum512(float v, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < RESID_THREADS / 64; ++w) t += red[w];
    return t;
}

template <int MAXV>
__global__ __launch_bounds__(RESID_THREADS) void epi_resid_kernel(const float* __restrict__ partial, int split,
                                                                   size_t slice_stride, const float* __restrict__ resid,
                                                                   float* __restrict__ x_out,
                                                                   const bf16_t* __restrict__ ln_w,
                                                                   bf16_t* __restrict__ r_out, int d, float eps,
                                                                   const int* __restrict__ row_live) {
    __shared__ float red[RESID_THREADS / 64];
    const size_t row = blockIdx.x;
    if (row_live && row_live[row] < 0) return;  // padding row
    const int nv = d / 4;
    f32x4 v[MAXV];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
        const int i = threadIdx.x + j * RESID_THREADS;
        if (i < nv) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
            if (resid) a = reinterpret_cast<const f32x4*>(resid + row * d)[i];
            const f32x4* p = reinterpret_cast<const f32x4*>(partial + row * d) + i;
            const size_t st = slice_stride / 4;
            int s = 0;
            for (; s + 4 <= split; s += 4) {  // four independent loads in flight, summed in slice order
                const f32x4 p0 = p[(size_t)s * st], p1 = p[(size_t)(s + 1) * st], p2 = p[(size_t)(s + 2) * st],
                            p3 = p[(size_t)(s + 3) * st];
                a += p0;
                a += p1;
                a += p2;
                a += p3;
            }
            for (; s < split; ++s) a += p[(size_t)s * st];
            reinterpret_cast<f32x4*>(x_out + row * d)[i] = a;
            v[j] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    if (ln_w == nullptr) return;
    const float inv = rsqrtf(block_sum512(ss, red) / (float)d + eps);
    const u32x2* wr = reinterpret_cast<const u32x2*>(ln_w);
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
        const int i = threadIdx.x + j * RESID_THREADS;
        if (i < nv) {
            const u32x2 g = wr[i];
            u32x2 o;
            o.x = pack_bf16x2(v[j].x * inv * __uint_as_float(g.x << 16), v[j].y * inv * __uint_as_float(g.x & 0xffff0000u));
            o.y = pack_bf16x2(v[j].z * inv * __uint_as_float(g.y << 16), v[j].w * inv * __uint_as_float(g.y & 0xffff0000u));
            reinterpret_cast<u32x2*>(r_out + row * d)[i] = o;
        }
    }
}

// ------------------------------------------------------------------ sum K slices + bias + RoPE + KV append
// Grid (token row, chunk of work items).  Work item = four consecutive rotate-half pairs
// (j..j+3, j+hd/2..j+hd/2+3) of one head: two 16-byte loads per K slice.  v heads are copied
// unrotated.  q goes to q_out[row]; k, v go to the token's slot in the paged pools.
__global__ __launch_bounds__(ROW_THREADS) void epi_qkv_kernel(const float* __restrict__ partial, int split,
                                                               size_t slice_stride, const bf16_t* __restrict__ bias,
                                                               const int* __restrict__ tok_pos,
                                                               const int* __restrict__ tok_slot,
                                                               const float2* __restrict__ rope, int max_pos,
                                                               bf16_t* __restrict__ q_out,
                                                               bf16_t* __restrict__ k_pool, bf16_t* __restrict__ v_pool,
                                                               int n_q, int n_kv, int hd) {
    const size_t row = blockIdx.x;
    const int half = hd / 2, per_head = half / 4;
    const int n_items = (n_q + 2 * n_kv) * per_head;
    const int it = blockIdx.y * ROW_THREADS + threadIdx.x;
    if (it >= n_items) return;
    const int pos = tok_pos[row], slot = tok_slot[row];
    const int width = (n_q + 2 * n_kv) * hd;
    const int head = it / per_head, j = (it % per_head) * 4;
    const int c0 = head * hd + j, c1 = c0 + half;
    if (pos < 0 || slot < 0) {  // padding row: defined q (zero), no cache write, partial sums not read
        if (head < n_q) {
            const u32x2 z = {0u, 0u};
            *reinterpret_cast<u32x2*>(q_out + row * (size_t)(n_q * hd) + c0) = z;
            *reinterpret_cast<u32x2*>(q_out + row * (size_t)(n_q * hd) + c1) = z;
        }
        return;
    }
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
    const float* p = partial + row * width;
    for (int s = 0; s < split; ++s) {
        a += *reinterpret_cast<const f32x4*>(p + s * slice_stride + c0);
        b += *reinterpret_cast<const f32x4*>(p + s * slice_stride + c1);
    }
    if (bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] += bf16_to_f32(bias[c0 + e]);
            b[e] += bf16_to_f32(bias[c1 + e]);
        }
    }
    if (head < n_q + n_kv) {
        // positions past the table are the caller's error; clamp so that the read stays in bounds
        const float2* cs = rope + (size_t)(pos < max_pos ? pos : max_pos - 1) * half + j;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float2 t = cs[e];
            const float ra = a[e] * t.x - b[e] * t.y;
            const float rb = b[e] * t.x + a[e] * t.y;
            a[e] = ra;
            b[e] = rb;
        }
    }
    u32x2 wa, wb;
    wa.x = pack_bf16x2(a.x, a.y);
    wa.y = pack_bf16x2(a.z, a.w);
    wb.x = pack_bf16x2(b.x, b.y);
    wb.y = pack_bf16x2(b.z, b.w);
    const int page = slot / LAPS_PAGE, off = slot % LAPS_PAGE;
    if (head < n_q) {
        *reinterpret_cast<u32x2*>(q_out + row * (size_t)(n_q * hd) + c0) = wa;
        *reinterpret_cast<u32x2*>(q_out + row * (size_t)(n_q * hd) + c1) = wb;
    } else if (head < n_q + n_kv) {
        const int g = head - n_q;
        bf16_t* dst = k_pool + (((size_t)page * n_kv + g) * LAPS_PAGE + off) * hd;
        *reinterpret_cast<u32x2*>(dst + j) = wa;
        *reinterpret_cast<u32x2*>(dst + j + half) = wb;
    } else {
        const int g = head - n_q - n_kv;
        bf16_t* dst = v_pool + ((size_t)page * n_kv + g) * hd * LAPS_PAGE + off;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            dst[(size_t)(j + e) * LAPS_PAGE] = f32_to_bf16(a[e]);
            dst[(size_t)(j + half + e) * LAPS_PAGE] = f32_to_bf16(b[e]);
        }
    }
}

// ------------------------------------------------------------------ sum K slices + SwiGLU
// Packed gate/up columns: block b of 64 columns = gate cols [32b, 32b+32) then up cols [32b, 32b+32).
__global__ __launch_bounds__(ROW_THREADS) void epi_swiglu_kernel(const float* __restrict__ partial, int split,
                                                                  size_t slice_stride, bf16_t* __restrict__ act,
                                                                  int inter, const int* __restrict__ row_live) {
    const size_t row = blockIdx.x;
    const int width = 2 * inter;
    if (row_live && row_live[row] < 0) return;  // padding row
    {
        const int c4 = blockIdx.y * ROW_THREADS + threadIdx.x;
        if (c4 >= inter / 4) return;
        const int c = c4 * 4;
        const int blk = c / 32, in = c % 32;
        const size_t gcol = (size_t)blk * 64 + in;
        f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < split; ++s) {
            const float* p = partial + s * slice_stride + row * width;
            g += *reinterpret_cast<const f32x4*>(p + gcol);
            u += *reinterpret_cast<const f32x4*>(p + gcol + 32);
        }
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = g[e] / (1.f + __expf(-g[e])) * u[e];
        u32x2 w;
        w.x = pack_bf16x2(o.x, o.y);
        w.y = pack_bf16x2(o.z, o.w);
        *reinterpret_cast<u32x2*>(act + row * inter + c) = w;
    }
}

// ------------------------------------------------------------------ gate/up interleave
__global__ void pack_gate_up_kernel(const u32x4* __restrict__ wg, const u32x4* __restrict__ wu, u32x4* __restrict__ dst,
                                    int inter, int row_vecs) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)2 * inter * row_vecs;
    if (i >= total) return;
    const size_t drow = i / row_vecs, v = i % row_vecs;
    const size_t blk = drow / 64, in = drow % 64;
    const size_t srow = blk * 32 + (in % 32);
    dst[i] = (in < 32 ? wg : wu)[srow * row_vecs + v];
}

// ------------------------------------------------------------------ token-major K/V <-> pools
template <bool SCATTER>
__global__ void kv_move_kernel(int n_seq, int n_tokens, const int* __restrict__ cu, const int* __restrict__ start_pos,
                               const int* __restrict__ page_table, int max_pages, bf16_t* __restrict__ k_tok,
                               bf16_t* __restrict__ v_tok, bf16_t* __restrict__ k_pool, bf16_t* __restrict__ v_pool,
                               int n_kv, int hd, int n_pool_pages) {
    const int tok = blockIdx.x;
    if (tok >= n_tokens) return;
    int lo = 0, hi = n_seq;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= tok) lo = mid; else hi = mid;
    }
    const int pos = start_pos[lo] + (tok - cu[lo]);
    if (pos < 0 || pos / LAPS_PAGE >= max_pages) return;  // outside the table
    const int page = page_table[(size_t)lo * max_pages + pos / LAPS_PAGE], off = pos % LAPS_PAGE;
    if (page < 0 || page >= n_pool_pages) return;  // unset table entry, or not a page of the pool
    for (int i = threadIdx.x; i < n_kv * hd; i += blockDim.x) {
        const int g = i / hd, e = i % hd;
        const size_t kp = (((size_t)page * n_kv + g) * LAPS_PAGE + off) * hd + e;
        const size_t vp = (((size_t)page * n_kv + g) * hd + e) * LAPS_PAGE + off;
        const size_t tp = (size_t)tok * n_kv * hd + i;
        if (SCATTER) {
            k_pool[kp] = k_tok[tp];
            v_pool[vp] = v_tok[tp];
        } else {
            k_tok[tp] = k_pool[kp];
            v_tok[tp] = v_pool[vp];
        }
    }
}

// Metadata of one captured bucket, from what the caller staged for its first n_real slots: lengths
// clamped to [0, len_bucket], prefix lengths to >= 0, the other slots empty, and the sequences packed
// one after the other (row_start = running sum of the clamped lengths, so the total never exceeds the
// graph's depth * len_bucket rows whatever the caller's arrays hold); then the attention's work-item table
// for those lengths.  One workgroup; thread t owns a run of consecutive slots.
constexpr int META_THREADS = 256;
__global__ __launch_bounds__(META_THREADS) void stage_meta_kernel(const StageArgs a) {
    __shared__ int sums[META_THREADS];
    __shared__ int carry;
    const int t = threadIdx.x;
    const int depth = a.depth;
    const int per = (depth + META_THREADS - 1) / META_THREADS;
    const int lo = t * per, hi = (lo + per < depth) ? lo + per : depth;
    auto len_of = [&](int i) {
        int l = i < a.n_real ? a.seq_len[i] : 0;
        l = l > a.len_bucket ? a.len_bucket : l;
        return l < 0 ? 0 : l;
    };
    int mine = 0;
    for (int i = lo; i < hi; ++i) mine += len_of(i);
    sums[t] = mine;
    __syncthreads();
    for (int o = 1; o < META_THREADS; o <<= 1) {  // inclusive scan of the per-thread sums
        const int v = (t >= o) ? sums[t - o] : 0;
        __syncthreads();
        sums[t] += v;
        __syncthreads();
    }
    int run = sums[t] - mine;
    for (int i = lo; i < hi; ++i) {
        const int l = len_of(i);
        a.row_start_out[i] = run;
        a.seq_len_out[i] = l;
        a.new_len_out[i] = l;
        const int pf = i < a.n_real ? a.prefix_len[i] : 0;
        a.prefix_out[i] = pf < 0 ? 0 : pf;
        run += l;
    }
    if (t == META_THREADS - 1) a.row_start_out[depth] = sums[t];
    __syncthreads();   // the lengths written above are read below by other threads of this workgroup
    laps_dev_attn_sched(a.new_len_out, depth, a.group, a.rows_per_wg, a.tile_start, a.item_seq, a.max_items, sums, &carry);
}

// One workgroup per graph row; see StageArgs.  Runs after stage_meta_kernel on the same stream.
__global__ __launch_bounds__(ROW_THREADS) void stage_rows_kernel(const StageArgs a) {
    __shared__ float red[ROW_THREADS / 64];
    __shared__ int live;
    const int row = blockIdx.x;
    {   // this workgroup's share of the page-table copy
        const int total = a.depth * a.max_pages, n_src = a.n_real * a.max_pages;
        const int chunk = (total + (int)gridDim.x - 1) / (int)gridDim.x;
        const int end = (row + 1) * chunk < total ? (row + 1) * chunk : total;
        for (int i = row * chunk + threadIdx.x; i < end; i += ROW_THREADS) a.page_table_out[i] = i < n_src ? a.page_table[i] : 0;
    }
    if (threadIdx.x == 0) {
        int pos, slot;   // lengths, prefixes and row offsets as clamped by stage_meta_kernel; page ids from the caller's table
        token_meta(row, a.depth, a.row_start_out, a.seq_len_out, a.prefix_out, a.page_table, a.max_pages, a.n_pool_pages,
                   &pos, &slot);
        a.tok_pos[row] = pos;
        a.tok_slot[row] = slot;
        live = pos >= 0;
    }
    const f32x4* src = reinterpret_cast<const f32x4*>(a.x_in + (size_t)row * a.d);
    if (a.x_rows != nullptr && row < a.n_rows) {
        src = reinterpret_cast<const f32x4*>(a.x_rows + (size_t)row * a.d);
        f32x4* dst = reinterpret_cast<f32x4*>(a.x_in + (size_t)row * a.d);
        if (src != dst)
            for (int i = threadIdx.x; i < a.d / 4; i += ROW_THREADS) dst[i] = src[i];
    }
    __syncthreads();
    if (!live) return;   // padding row: nothing reads its normed row
    rmsnorm_row(src, a.ln_w, a.r0 + (size_t)row * a.d, a.d, a.eps, red);
}

}  // namespace

int laps_launch_stage(const StageArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(stage_meta_kernel, dim3(1), dim3(META_THREADS), 0, s, a);
    LAPS_LAUNCH_CHECK();
    hipLaunchKernelGGL(stage_rows_kernel, dim3(a.depth * a.len_bucket), dim3(ROW_THREADS), 0, s, a);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_rope_table(float2* table, int max_pos, int head_dim, float theta, hipStream_t s) {
    const int half = head_dim / 2;
    const int n = max_pos * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, table, max_pos, half, (double)theta,
                       head_dim);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_prep(int n_rows, int n_seq, const int* row_start, const int* seq_len, const int* prefix_len,
                     const int* page_table, int max_pages, int n_pool_pages, int* new_len_out, int* tok_pos,
                     int* tok_slot, hipStream_t s) {
    const int n = n_rows > n_seq ? n_rows : n_seq;
    hipLaunchKernelGGL(prep_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n_rows, n_seq, row_start, seq_len,
                       prefix_len, page_table, max_pages, n_pool_pages, new_len_out, tok_pos, tok_slot);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_rmsnorm(const float* x, const bf16_t* w, bf16_t* out, int rows, int d, float eps, const int* row_live,
                        hipStream_t s) {
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(ROW_THREADS), 0, s, x, w, out, d, eps, row_live);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_epi_resid(const float* partial, int split, const float* resid, float* x_out, const bf16_t* ln_w,
                          bf16_t* r_out, int rows, int d, float eps, const int* row_live, hipStream_t s) {
    const size_t stride = (size_t)rows * d;
    if (d <= 4 * RESID_THREADS * 1)
        hipLaunchKernelGGL(epi_resid_kernel<1>, dim3(rows), dim3(RESID_THREADS), 0, s, partial, split, stride, resid,
                           x_out, ln_w, r_out, d, eps, row_live);
    else if (d <= 4 * RESID_THREADS * 4)
        hipLaunchKernelGGL(epi_resid_kernel<4>, dim3(rows), dim3(RESID_THREADS), 0, s, partial, split, stride, resid,
                           x_out, ln_w, r_out, d, eps, row_live);
    else {
        laps_set_error("row width %d too large for the fused residual + norm kernel (max %d)", d, 4 * RESID_THREADS * 4);
        return LAPS_EINVAL;
    }
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_epi_qkv(const float* partial, int split, const bf16_t* bias, const int* tok_pos, const int* tok_slot,
                        const float2* rope, int max_pos, bf16_t* q_out, bf16_t* k_pool, bf16_t* v_pool, int rows,
                        int n_q, int n_kv, int hd, hipStream_t s) {
    const size_t stride = (size_t)rows * (n_q + 2 * n_kv) * hd;
    const int n_items = (n_q + 2 * n_kv) * (hd / 8);
    hipLaunchKernelGGL(epi_qkv_kernel, dim3(rows, (n_items + ROW_THREADS - 1) / ROW_THREADS), dim3(ROW_THREADS), 0, s,
                       partial, split, stride, bias, tok_pos, tok_slot, rope, max_pos, q_out, k_pool, v_pool, n_q, n_kv,
                       hd);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_epi_swiglu(const float* partial, int split, bf16_t* act, int rows, int inter, const int* row_live,
                           hipStream_t s) {
    const size_t stride = (size_t)rows * 2 * inter;
    hipLaunchKernelGGL(epi_swiglu_kernel, dim3(rows, (inter / 4 + ROW_THREADS - 1) / ROW_THREADS), dim3(ROW_THREADS), 0,
                       s, partial, split, stride, act, inter, row_live);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_pack_gate_up(const bf16_t* wg, const bf16_t* wu, bf16_t* dst, int inter, int d, hipStream_t s) {
    const int row_vecs = d / 8;
    const size_t total = (size_t)2 * inter * row_vecs;
    hipLaunchKernelGGL(pack_gate_up_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<const u32x4*>(wg), reinterpret_cast<const u32x4*>(wu),
                       reinterpret_cast<u32x4*>(dst), inter, row_vecs);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}

int laps_launch_kv_move(bool scatter, int n_seq, int n_tokens, const int* cu, const int* start_pos,
                        const int* page_table, int max_pages, bf16_t* k_tok, bf16_t* v_tok, bf16_t* k_pool,
                        bf16_t* v_pool, int n_kv, int hd, int n_pool_pages, hipStream_t s) {
    if (n_tokens == 0) return LAPS_OK;
    if (scatter)
        hipLaunchKernelGGL(kv_move_kernel<true>, dim3(n_tokens), dim3(256), 0, s, n_seq, n_tokens, cu, start_pos,
                           page_table, max_pages, k_tok, v_tok, k_pool, v_pool, n_kv, hd, n_pool_pages);
    else
        hipLaunchKernelGGL(kv_move_kernel<false>, dim3(n_tokens), dim3(256), 0, s, n_seq, n_tokens, cu, start_pos,
                           page_table, max_pages, k_tok, v_tok, k_pool, v_pool, n_kv, hd, n_pool_pages);
    LAPS_LAUNCH_CHECK();
    return LAPS_OK;
}
