// Host-side launch interface of the gfx950 kernels.  Every function validates nothing:
// the runtime (shard.cpp) checks shapes before it calls them.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "device_utils.hpp"

namespace shk {

// Element types inside the library.  bf16 only exists at the boundary: shard_create converts
// bf16 matrices to IEEE half once (launch_bf16_to_f16).
enum DType { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };

// Kernel timing.  While the runtime has a timer installed on the calling thread, every launch
// asks it for a start/stop event pair and attaches the pair to its own dispatch, so the pair
// reads the kernel's execution time (what a profiler's kernel trace reports) without the gap
// between launches.  Without a timer the launch is an ordinary one.
struct LaunchTimer {
    bool (*next)(void* ctx, hipEvent_t* start, hipEvent_t* stop) = nullptr;
    void* ctx = nullptr;
};
extern thread_local LaunchTimer g_launch_timer;  // defined by the runtime

template <typename... P, typename... A>
inline void launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t st, A... args) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (g_launch_timer.next && g_launch_timer.next(g_launch_timer.ctx, &e0, &e1))
        hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), st, e0, e1, 0u, static_cast<P>(args)...);
    else
        hipLaunchKernelGGL(kernel, grid, block, lds, st, static_cast<P>(args)...);
}

// One layer's paged KV cache.  Element (page p, kv head h, slot s, e) of K or V lives at
// ((p * hkv + h) * page + s) * dh + e; token u of sequence q is in page
// block_table[q * max_pages + u / page], slot u % page.
struct KvView {
    void* k;
    void* v;
    const int32_t* block_table;
    int32_t max_pages, page, hkv, dh;
    uint32_t page_magic;   // ceil(2^32 / page) for page >= 2: u / page == mulhi(u, page_magic) while u * page < 2^32
};

// Page number and slot of token position u, without an integer division.
__device__ __forceinline__ void kv_split(const KvView& kv, int u, int* pg, int* slot) {
    const uint32_t q = kv.page == 1 ? static_cast<uint32_t>(u) : __umulhi(static_cast<uint32_t>(u), kv.page_magic);
    *pg = static_cast<int>(q);
    *slot = u - static_cast<int>(q) * kv.page;
}
// Row (in units of dh elements) of token u of the sequence whose block-table row is bt, kv head hk.
// Two forms of the same index: kv_row finds the page with a multiply-high, kv_row_div with the
// compiler's division sequence.  Which one is faster depends on the kernel around it (the
// division's longer address computation happens to be scheduled further ahead of the loads
// that need it); each kernel uses the form that measured faster.
__device__ __forceinline__ size_t kv_row_div(const KvView& kv, const int32_t* bt, int u, int hk) {
    return (static_cast<size_t>(bt[u / kv.page]) * kv.hkv + hk) * kv.page + u % kv.page;
}
__device__ __forceinline__ size_t kv_row(const KvView& kv, const int32_t* bt, int u, int hk) {
    int pg, slot;
    kv_split(kv, u, &pg, &slot);
    return (static_cast<size_t>(bt[pg]) * kv.hkv + hk) * kv.page + slot;
}

enum Epilogue {
    EPI_QKV = 0,     // RoPE on q,k; q -> q buffer (fp32); k,v -> cache pages
    EPI_RESID = 1,   // out = resid + acc   (fp32)
    EPI_SWIGLU = 2,  // rows (2f, 2f+1) = (gate_f, up_f): out[f] = silu(gate) * up
    EPI_STORE = 3,   // out = acc   (fp32; decode path only: the LM head)
    EPI_PARTIAL = 4  // out = acc   (fp32; prefill GEMM only: one K slice's partial sums)
};

// y = W x for a few activation rows (decode): W [N, K] row-major (dtype wt), x fp32 [nb, K].
struct DecodeLinear {
    const void* W;
    int32_t N, K;
    int32_t wt;            // DType of W
    int32_t nb;            // activation rows, 1..8 (matrix-core variant: 1..16)
    const float* x;        // [nb, K]
    const float* gain;     // non-null: RMSNorm(x; gain, eps) is applied to x on the fly
    float eps;
    int32_t epi;
    // EPI_RESID
    const float* resid;    // [nb, N]
    float* out;            // [nb, N]  (EPI_SWIGLU: [nb, N/2])
    // EPI_QKV
    float* q;              // [nb, hq*dh]
    int32_t hq;
    KvView kv;
    const float2* rope;    // [max_seq_len, dh/2] (cos, sin)
    // matrix-core variant (launch_decode_linear_mfma): half weights, up to 16 rows
    const void* xb;        // [nb, K] half activations
    void* out_b;           // EPI_SWIGLU output [nb, N/2] half
    int32_t norm_xb;       // non-zero: xb is un-normalised; scale row b of the result by
                           // rsqrt(mean_k xb[b][k]^2 + eps) (RMSNorm with the gain folded into W)
    void* out_h;           // EPI_RESID: non-null -> also store the result as half [nb, N]
    uint32_t* oflow;       // set to 1 when a value stored as half leaves half's range (16-bit weights only)
};
void launch_decode_linear(const DecodeLinear& a, const SeqBatch& sb, hipStream_t st);
// same contract with xb/out_b; requires wt == DT_F16, nb <= 16, K % 64 == 0, gain == null
void launch_decode_linear_mfma(const DecodeLinear& a, const SeqBatch& sb, hipStream_t st);

struct DecodeAttn {
    const float* q;        // [nb, hq*dh], already rotated
    void* o;               // [nb, hq*dh] in o_dtype
    int32_t o_dtype;
    int32_t nb, hq;
    int32_t kv_dtype;
    KvView kv;
    int32_t nsplit;        // context splits per (sequence, head)
    float* part_o;         // [nb*hq, nsplit, dh]
    float* part_ml;        // [nb*hq, nsplit, 2]
};
void launch_decode_attn(const DecodeAttn& a, const SeqBatch& sb, hipStream_t st);
// context tokens one workgroup of the decode attention kernel covers per trip
int decode_attn_heads_per_group(int kv_dtype, int dh, int hq, int hkv);
int decode_attn_tokens_per_trip(int kv_dtype, int dh, int hq, int hkv);
int decode_attn_target_workgroups(int kv_dtype, int dh, int hq, int hkv);
int decode_attn_single_pass_ctx(int kv_dtype, int dh, int hq, int hkv);

// rows of x [M, d] fp32 -> RMSNorm -> out [M, d] in out_dtype
void launch_rmsnorm(const float* x, const float* gain, float eps, void* out, int32_t out_dtype,
                    int32_t M, int32_t d, hipStream_t st);

// C = A W^T for many activation rows (prefill): A [M, K] and W [N, K] in dtype `dt`.
struct PrefillGemm {
    const void* A;
    const void* W;
    int32_t M, N, K;
    int32_t dt;            // DType of A and W
    int32_t epi;
    int32_t T;             // tokens per sequence: row m is (sequence m / T, token m % T)
    // EPI_RESID: fp32
    const float* resid;    // [M, N]
    float* out;            // [M, N]
    // EPI_SWIGLU: out_act [M, N/2] in dtype dt
    void* out_act;
    // EPI_QKV
    float* q;              // [M, hq*dh] fp32
    int32_t hq;
    KvView kv;
    const float2* rope;
    // EPI_RESID with few output tiles: scratch for split-K partial sums (may be null) and its
    // capacity in floats; kslices is set by the launcher
    float* part;
    size_t part_cap;
    int32_t kslices;
    uint32_t* oflow;       // set to 1 when a value stored as half leaves half's range (half operands only)
};
void launch_prefill_gemm(const PrefillGemm& a, const SeqBatch& sb, hipStream_t st);

// Which kernel variant a launch takes - pure host functions of the shape, the same ones the
// launchers call.  Each returns an index into its family's name table (name(id) is null past
// the end of the table).
int choose_prefill_gemm(int dt, int M, int N, int K, int epi, bool has_part, size_t part_cap, int* kslices);
const char* prefill_gemm_variant_name(int id);
int choose_decode_linear(int wt, int nb, int N, int K);
const char* decode_linear_variant_name(int id);
int choose_decode_linear_mfma(int N, int K, int* rows_wg);
const char* decode_linear_mfma_variant_name(int id);

struct PrefillAttn {
    const float* q;        // [B*T, hq*dh] fp32, rotated
    void* o;               // [B*T, hq*dh] in out_dtype
    int32_t out_dtype;
    int32_t B, T, hq;
    int32_t kv_dtype;
    KvView kv;
};
void launch_prefill_attn(const PrefillAttn& a, const SeqBatch& sb, hipStream_t st);

// W[n][k] *= gain[k] for a half matrix [N, K] (RMSNorm gains folded into the matrix that
// consumes the normalised vector); *overflow is set when a product leaves half's range.
void launch_scale_columns_f16(void* W, const float* gain, int32_t N, int32_t K, uint32_t* overflow, hipStream_t st);
// out[i] = half(x[i]), i < n (n a multiple of 4); *oflow is set when a value leaves half's range
void launch_to_half(const float* x, void* out, size_t n, uint32_t* oflow, hipStream_t st);

// First failure of a one-time kernel attribute call (the opt-in to more than 64 KB of LDS per
// workgroup), hipSuccess if none: the runtime reports it instead of a later launch error.
hipError_t kernel_attribute_error();
void note_kernel_attribute(hipError_t e);
// test hook: pretend such a call failed (true) / forget the pretended failure (false)
void inject_kernel_attribute_error(bool on);

// In place: n bf16 values -> n IEEE half values (round to nearest; exact for every bf16 in
// half's normal range).  *overflow is set when a finite value exceeds half's range.
void launch_bf16_to_f16(void* buf, size_t n, uint32_t* overflow, hipStream_t st);

// block_table[idx[i]] = val[i] for i < n (n <= 128), stream-ordered.
struct TableUpdate {
    int32_t n;
    int32_t idx[128];
    int32_t val[128];
};
void launch_table_update(int32_t* table, const TableUpdate& u, hipStream_t st);

// x_out[i, :] = table[ids[i], :] widened to fp32 (table [V, d] in dtype dt).  Ids come either
// by value (n <= 128) or from device memory; an id outside [0, V) is clamped and *bad is set.
struct TokenIds {
    int32_t n;
    int32_t id[128];
};
void launch_embed(const void* table, int32_t dt, int32_t V, int32_t d, const TokenIds* by_value, const int32_t* ids_dev,
                  int32_t n, float* x_out, uint32_t* bad, hipStream_t st);

// out[i] = index of the largest of logits[i, 0..V) (the lowest index among equals; NaNs are
// never chosen unless the whole row is NaN, which gives 0).
void launch_argmax(const float* logits, int32_t n, int32_t V, int32_t* out, hipStream_t st);

}  // namespace shk
