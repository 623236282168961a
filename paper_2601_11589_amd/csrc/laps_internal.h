// Internal declarations shared by the HIP translation units of liblaps (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/laps.h"

typedef unsigned short bf16_t;  // storage: upper half of a float32
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static __device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((unsigned)b) << 16); }
static __device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    __bf16 h = (__bf16)f;  // v_cvt_pk_bf16_f32: round-to-nearest-even
    return __builtin_bit_cast(bf16_t, h);
}
static __device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    return (unsigned)f32_to_bf16(lo) | ((unsigned)f32_to_bf16(hi) << 16);
}

void laps_set_error(const char* fmt, ...);
#define LAPS_HIP(call)                                                                         \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess) {                                                                \
            laps_set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return LAPS_EHIP;                                                                  \
        }                                                                                      \
    } while (0)
#define LAPS_LAUNCH_CHECK()                                                                    \
    do {                                                                                       \
        hipError_t e_ = hipGetLastError();                                                     \
        if (e_ != hipSuccess) {                                                                \
            laps_set_error("kernel launch failed: %s (%s:%d)", hipGetErrorString(e_), __FILE__, __LINE__); \
            return LAPS_EHIP;                                                                  \
        }                                                                                      \
    } while (0)

// ----------------------------------------------------------------------------- GEMM
// C = A[M,K] * W[N,K]^T, bf16 operands, fp32 accumulation, K-split into `split` slices.
enum GemmEpi {
    EPI_PARTIAL = 0,  // out_f32[split][M][N] raw partial sums
    EPI_RESID = 1,    // out_f32[M][N] = resid[M][N] + C              (single K slice only)
    EPI_SWIGLU = 2,   // out_bf16[M][N/2] = silu(gate) * up on interleaved columns (single K slice only)
};
struct GemmPlan {
    int cfg;          // tile shape index (see kTiles in gemm.hip)
    int split;        // K slices
    int k_per_split;  // multiple of 64
    int epi;          // epilogue the launch will apply: the requested one if split == 1, else EPI_PARTIAL
    int ws;           // weight slabs kept in flight per workgroup (register sets): 1 or 2
};
GemmPlan laps_gemm_plan(int m, int n, int k, int force_split, int want_epi);
size_t laps_gemm_partial_bytes(int m, int n, int k);
void laps_gemm_tile_dims(int cfg, int* bm, int* bn);   // rows and columns of tile shape `cfg` (0, 0 if unknown)
// row_live: NULL, or m entries; a negative entry marks a padding row.  Output rows of padding are unspecified:
// the skinny tiles do not load them (they compute with zeros), and a row tile of padding only is skipped.
int laps_gemm_launch(const GemmPlan& p, const bf16_t* a, const bf16_t* w, int m, int n, int k, float* out_f32,
                     const float* resid, bf16_t* out_bf16, const int* row_live, hipStream_t s);

// ----------------------------------------------------------------------------- element-wise / epilogues
int laps_launch_rope_table(float2* table, int max_pos, int head_dim, float theta, hipStream_t s);
// n_pool_pages (here, in the K/V movers and in the attention): page ids outside [0, n_pool_pages) are treated as
// unset entries - no cache write, no wild read.  INT_MAX when the caller has not said how many pages its pools hold.
int laps_launch_prep(int n_rows, int n_seq, const int* row_start, const int* seq_len, const int* prefix_len,
                     const int* page_table, int max_pages, int n_pool_pages, int* new_len_out, int* tok_pos,
                     int* tok_slot, hipStream_t s);
// row_live (here and below): NULL, or one entry per row; rows with a negative entry are padding and are skipped.
int laps_launch_rmsnorm(const float* x, const bf16_t* w, bf16_t* out, int rows, int d, float eps, const int* row_live,
                        hipStream_t s);
// x_out = resid + sum_s partial[s]; if ln_w: r_out = rmsnorm(x_out; ln_w) in bf16.
int laps_launch_epi_resid(const float* partial, int split, const float* resid, float* x_out, const bf16_t* ln_w,
                          bf16_t* r_out, int rows, int d, float eps, const int* row_live, hipStream_t s);
int laps_launch_epi_qkv(const float* partial, int split, const bf16_t* bias, const int* tok_pos, const int* tok_slot,
                        const float2* rope, int max_pos, bf16_t* q_out, bf16_t* k_pool, bf16_t* v_pool, int rows,
                        int n_q, int n_kv, int hd, hipStream_t s);
int laps_launch_epi_swiglu(const float* partial, int split, bf16_t* act, int rows, int inter, const int* row_live,
                           hipStream_t s);
int laps_launch_pack_gate_up(const bf16_t* wg, const bf16_t* wu, bf16_t* dst, int inter, int d, hipStream_t s);
int laps_launch_kv_move(bool scatter, int n_seq, int n_tokens, const int* cu, const int* start_pos,
                        const int* page_table, int max_pages, bf16_t* k_tok, bf16_t* v_tok, bf16_t* k_pool,
                        bf16_t* v_pool, int n_kv, int hd, int n_pool_pages, hipStream_t s);
// Graph staging, two launches that leave a captured stack nothing to prepare:
// (1) one workgroup: clamped lengths / prefixes of `depth` slots (the first n_real from the caller's device arrays,
//     the rest empty), packed row offsets row_start_out[depth + 1], and the attention's work-item table for them;
// (2) one workgroup per graph row: token position and cache slot (as laps_launch_prep), the row's input copied from
//     x_rows (rows below n_rows; NULL: the graph's input rows are used as they are) into x_in, its RMSNorm with the
//     first layer's gain into r0, and a share of the page-table copy (entries past n_real rows become 0).
struct StageArgs {
    const int *seq_len, *prefix_len, *page_table;   // caller's device arrays: [n_real], [n_real], [n_real][max_pages]
    const float* x_rows;                            // caller's packed input rows or NULL
    int n_real, n_rows, depth, len_bucket, max_pages, n_pool_pages;
    int group, rows_per_wg, max_items;              // attention blocking of the graph's shape
    int *seq_len_out, *prefix_out, *row_start_out, *page_table_out;   // the graph's staging block
    int *new_len_out, *tok_pos, *tok_slot, *tile_start, *item_seq;    // the graph's workspace
    float* x_in;
    const bf16_t* ln_w;
    bf16_t* r0;
    int d;
    float eps;
};
int laps_launch_stage(const StageArgs& a, hipStream_t s);

// Work-item table of the attention for one batch: per-sequence number of query-row blocks, their exclusive prefix
// sum (tile_start[n_seq + 1]) and the sequence of every work item.  Runs in ONE workgroup of 256 threads; buf holds
// 256 ints and carry one int of LDS.  Shared by the stand-alone scheduling kernel and the staging kernel of graphs.
static __device__ __forceinline__ void laps_dev_attn_sched(const int* __restrict__ new_len, int n_seq, int group,
                                                           int rows_per_wg, int* __restrict__ tile_start,
                                                           int* __restrict__ item_seq, int max_items, int* buf,
                                                           int* carry) {
    if (threadIdx.x == 0) *carry = 0;
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
        const int c = *carry;
        if (i < n_seq) {
            const int first = c + buf[threadIdx.x] - v;
            tile_start[i] = first;
            // bound: lengths that disagree with the row offsets must not write past the table
            for (int k = 0; k < v && first + k < max_items; ++k) item_seq[first + k] = i;
        }
        __syncthreads();
        if (threadIdx.x == 255) *carry = c + buf[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) tile_start[n_seq] = *carry;
}

// ----------------------------------------------------------------------------- attention
// Both take the same (n_seq, n_tokens, max_pages): the blocking they derive from them must agree.
// `partial` (laps_attn_partial_bytes, 16-byte aligned) receives per-split results when the launch shape
// calls for splitting the key range; it may be NULL only if max_pages * 16 < 1024.
// tile_start: n_seq + 1 ints; item_seq: laps_attn_item_table_bytes (sequence of every row-block work item).
size_t laps_attn_partial_bytes(int hd, int max_pages);   // 0 when page tables this narrow never split
size_t laps_attn_item_table_bytes(int max_tokens, int max_seqs, int group);
// The blocking laps_launch_attn_sched / laps_launch_attention derive from a launch shape: query rows per workgroup,
// bound on the (sequence, row block) items, key-range splits (1 = none), fewest key tiles a split may get.
void laps_attn_plan(int n_seq, int n_tokens, int group, int n_kv, int max_pages, int* rows_per_wg, int* max_items,
                    int* n_split, int* min_tiles_per_split);
int laps_launch_attn_sched(const int* new_len, int n_seq, int n_tokens, int max_pages, int* tile_start, int* item_seq,
                           int n_q, int n_kv, hipStream_t s);
int laps_launch_attention(const bf16_t* q, bf16_t* out, const bf16_t* k_pool, const bf16_t* v_pool,
                          const int* row_start, const int* new_len, const int* prefix_len, const int* page_table,
                          int max_pages, int n_seq, int n_tokens, const int* tile_start, const int* item_seq,
                          float* partial, int n_q, int n_kv, int hd, int n_pool_pages, hipStream_t s);
