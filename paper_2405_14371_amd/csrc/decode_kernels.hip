// Autoregressive-phase kernels (EdgeShard Sec. 2: one token per iteration over the KV
// cache).  Every weight is read exactly once per step, so these kernels are HBM streams:
// 16-byte loads per lane, many independent loads in flight, fixed-order reductions.
#include "kernels.hpp"

#include <atomic>
#include <mutex>

namespace shk {

// ---------------------------------------------------------------------------------------
// Linear layer for nb <= NB activation rows.  One workgroup (256 threads) owns R
// consecutive output rows of W and the whole K extent: thread t covers the 16-byte chunks
// t, t+256, ... of every one of its R rows, so each chunk of x is loaded once and reused
// for R rows.  U chunks are fetched per trip so that U*R independent 16-byte loads per
// lane are in flight.  Partial sums are reduced across the wave with shuffles, across the
// four waves through LDS, always in the same order.
// ---------------------------------------------------------------------------------------
template <typename WT, int NB, int R, int U, bool ROT = false, int THREADS = 256>
__global__ __launch_bounds__(THREADS) void decode_linear_kernel(DecodeLinear a, SeqBatch sb) {
    constexpr int VEC = Elem<WT>::VEC;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.x * R;
    const int nchunk = a.K / VEC;
    // ROT: every workgroup starts its walk over K at its own 4 KB iteration.  With long rows
    // (K = 11008) this spreads the workgroups of a launch over the memory channels (+3..7 %);
    // with K = 4096 it gains nothing and costs a few instructions, so it is opt-in per shape.
    constexpr int WAVES = THREADS / 64;
    const int iters = (nchunk + THREADS - 1) / THREADS;
    const int rot = ROT ? static_cast<int>((blockIdx.x * 5u) % static_cast<unsigned>(iters)) * THREADS : 0;
    const WT* __restrict__ W = static_cast<const WT*>(a.W);
    const bool norm = a.gain != nullptr;

    __shared__ float s_red[WAVES][R * NB];
    __shared__ float s_ssq[WAVES][NB];

    float acc[R][NB];
    float ssq[NB];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[r][b] = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b) ssq[b] = 0.f;

    const WT* rowp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int n = min(row0 + r, a.N - 1);  // rows past N re-read the last row; never stored
        rowp[r] = W + static_cast<size_t>(n) * a.K;
    }

    // What the epilogue needs from memory is fetched NOW, by the threads that will run it, so that
    // the end of the workgroup is arithmetic and stores only: with every workgroup of a launch
    // resident at once they all finish together, and a chain of dependent loads there (residual;
    // position -> rotation table; block table -> page) was 1.6 - 3.3 us of every launch.
    typedef typename ActOf<WT>::type CT;  // cache element type
    float pre_resid = 0.f;                // EPI_RESID: the residual element of (row tid / NB, activation row tid % NB)
    float2 pre_cs = make_float2(1.f, 0.f);  // EPI_QKV: (cos, sin) of the pair this thread rotates
    size_t pre_at = 0;                    // EPI_QKV: element offset of the pair in the K or V pool
    if (a.epi == EPI_RESID) {
        if (tid < R * NB) {
            const int r = tid / NB, b = tid % NB, n = row0 + r;
            if (n < a.N && b < a.nb) pre_resid = a.resid[static_cast<size_t>(b) * a.N + n];
        }
    } else if (a.epi == EPI_QKV) {
        if (tid < (R / 2) * NB) {
            const int j = tid / NB, b = tid % NB, n0 = row0 + 2 * j;
            if (n0 < a.N && b < a.nb) {
                const int dh = a.kv.dh, nq = a.hq * dh, nk = a.kv.hkv * dh;
                const int pos = sb.pos[b], e = n0 % dh;
                if (n0 < nq + nk) pre_cs = a.rope[static_cast<size_t>(pos) * (dh / 2) + e / 2];
                if (n0 >= nq) {
                    const int hk = (n0 - nq - (n0 < nq + nk ? 0 : nk)) / dh;
                    pre_at = kv_row_div(a.kv, a.kv.block_table + static_cast<size_t>(sb.seq[b]) * a.kv.max_pages, pos, hk) * dh + e;
                }
            }
        }
    }

    for (int c0 = tid; c0 < nchunk; c0 += THREADS * U) {
        Vec16<WT> w[U][R];
        int cc[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + THREADS * u;
            ok[u] = c < nchunk;
            cc[u] = ok[u] ? c : c0;
            if constexpr (ROT) {  // walk K from a per-workgroup offset (a rotation of the chunk index)
                cc[u] += rot;
                if (cc[u] >= nchunk) cc[u] -= nchunk;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) w[u][r].load_stream(rowp[r] + static_cast<size_t>(cc[u]) * VEC);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float xv[NB][VEC];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float* xp = a.x + static_cast<size_t>(b < a.nb ? b : 0) * a.K + cc[u] * VEC;
#pragma unroll
                for (int e = 0; e < VEC; e += 4) {
                    const float4 t = *reinterpret_cast<const float4*>(xp + e);
                    xv[b][e] = t.x; xv[b][e + 1] = t.y; xv[b][e + 2] = t.z; xv[b][e + 3] = t.w;
                }
            }
            if (!ok[u]) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) xv[b][e] = 0.f;
            }
            if (norm) {
                float g[VEC];
#pragma unroll
                for (int e = 0; e < VEC; e += 4) {
                    const float4 t = *reinterpret_cast<const float4*>(a.gain + cc[u] * VEC + e);
                    g[e] = t.x; g[e + 1] = t.y; g[e + 2] = t.z; g[e + 3] = t.w;
                }
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        ssq[b] = fmaf(xv[b][e], xv[b][e], ssq[b]);
                        xv[b][e] *= g[e];
                    }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[r][b] = fmaf(w[u][r].v[e], xv[b][e], acc[r][b]);
        }
    }

#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float v = wave_sum_rows(acc[r][b]);
            if (lane == 0) s_red[wave][r * NB + b] = v;
        }
    if (norm) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float v = wave_sum_rows(ssq[b]);
            if (lane == 0) s_ssq[wave][b] = v;
        }
    }
    __syncthreads();
    // element idx = row * NB + activation row: the waves' partial sums in a fixed order, times the
    // RMSNorm factor of its activation row
    auto total = [&](int idx) {
        float v = 0.f;
        if constexpr (WAVES < 4) {
#pragma unroll
            for (int w = 0; w < WAVES; ++w) v += s_red[w][idx];
        } else {
#pragma unroll
            for (int w = 0; w < WAVES; w += 4) v += (s_red[w][idx] + s_red[w + 1][idx]) + (s_red[w + 2][idx] + s_red[w + 3][idx]);
        }
        if (norm) {
            const int b = idx % NB;
            float q = 0.f;
            if constexpr (WAVES < 4) {
#pragma unroll
                for (int w = 0; w < WAVES; ++w) q += s_ssq[w][b];
            } else {
#pragma unroll
                for (int w = 0; w < WAVES; w += 4) q += (s_ssq[w][b] + s_ssq[w + 1][b]) + (s_ssq[w + 2][b] + s_ssq[w + 3][b]);
            }
            const float ms = q / static_cast<float>(a.K);
            v *= 1.0f / sqrtf(ms + a.eps);
        }
        return v;
    };

    if (a.epi == EPI_RESID || a.epi == EPI_STORE) {
        if (tid < R * NB) {
            const int r = tid / NB, b = tid % NB, n = row0 + r;
            if (n < a.N && b < a.nb) a.out[static_cast<size_t>(b) * a.N + n] = pre_resid + total(tid);   // EPI_STORE: pre_resid is 0
        }
        return;
    }
    // the other epilogues work on row pairs (2j, 2j+1)
    if (tid >= (R / 2) * NB) return;
    const int j = tid / NB, b = tid % NB;
    const int n0 = row0 + 2 * j;
    if (n0 >= a.N || b >= a.nb) return;
    const float v0 = total((2 * j) * NB + b), v1 = total((2 * j + 1) * NB + b);
    if (a.epi == EPI_SWIGLU) {
        const int F = a.N / 2;
        a.out[static_cast<size_t>(b) * F + n0 / 2] = v0 / (1.0f + expf(-v0)) * v1;
        return;
    }
    // EPI_QKV
    const int dh = a.kv.dh, nq = a.hq * dh, nk = a.kv.hkv * dh;
    if (n0 < nq + nk) {  // q or k: rotate the pair
        const float r0 = v0 * pre_cs.x - v1 * pre_cs.y, r1 = v0 * pre_cs.y + v1 * pre_cs.x;
        if (n0 < nq) {
            a.q[static_cast<size_t>(b) * nq + n0] = r0;
            a.q[static_cast<size_t>(b) * nq + n0 + 1] = r1;
            return;
        }
        CT* kp = static_cast<CT*>(a.kv.k);
        kp[pre_at] = store_cast<CT>(r0, a.oflow);
        kp[pre_at + 1] = store_cast<CT>(r1, a.oflow);
        return;
    }
    CT* vp = static_cast<CT*>(a.kv.v);
    vp[pre_at] = store_cast<CT>(v0, a.oflow);
    vp[pre_at + 1] = store_cast<CT>(v1, a.oflow);
}

template <typename WT, int NB, int R, int U, bool ROT = false, int THREADS = 256>
static void launch_dl(const DecodeLinear& a, const SeqBatch& sb, hipStream_t st) {
    const int grid = (a.N + R - 1) / R;
    launch((decode_linear_kernel<WT, NB, R, U, ROT, THREADS>), dim3(grid), dim3(THREADS), 0, st, a, sb);
}

// (rows per workgroup, chunks in flight) from a sweep on MI355X over the Llama2 shapes:
// many small workgroups win; wide matrices like more rows per workgroup, bf16 rows
// (half the bytes) like more rows still.  The choice is a pure host function of the shape
// (choose_decode_linear), so that tests can ask which variant a shape lands on.
enum DlId { DL_NB1_WIDE, DL_NB1_LONGK, DL_NB1_SQUARE, DL_NB2, DL_NB4, DL_NB8, DL_ID_COUNT };
static const char* const DL_NAMES[2][DL_ID_COUNT] = {
    {"f32 stream nb1 r4 u1 t512 (N >= 8192)", "f32 stream nb1 r4 u2 rot (K > 8192)", "f32 stream nb1 r2 u4", "f32 stream nb2 r4 u2",
     "f32 stream nb4 r4 u2", "f32 stream nb8 r4 u1"},
    {"f16 stream nb1 r8 u1 t512 (N >= 8192)", "f16 stream nb1 r4 u1 t512 (K > 8192)", "f16 stream nb1 r4 u1 t512", "f16 stream nb2 r4 u2",
     "f16 stream nb4 r4 u2", "f16 stream nb8 r4 u1"}};
const char* decode_linear_variant_name(int id) {
    return id >= 0 && id < 2 * DL_ID_COUNT ? DL_NAMES[id / DL_ID_COUNT][id % DL_ID_COUNT] : nullptr;
}
// index into the name table: DL_ID_COUNT * (16-bit weights) + DlId
int choose_decode_linear(int wt, int nb, int N, int K) {
    int id;
    if (nb == 1) id = N >= 8192 ? DL_NB1_WIDE : (K > 8192 ? DL_NB1_LONGK : DL_NB1_SQUARE);
    else if (nb == 2) id = DL_NB2;
    else if (nb <= 4) id = DL_NB4;
    else id = DL_NB8;
    return (wt == DT_F32 ? 0 : DL_ID_COUNT) + id;
}

template <typename WT>
static void launch_dl_t(const DecodeLinear& a, const SeqBatch& sb, hipStream_t st) {
    constexpr bool f32 = sizeof(WT) == 4;
    switch (choose_decode_linear(a.wt, a.nb, a.N, a.K) % DL_ID_COUNT) {
        // threads per workgroup from the same sweep: 512 for the wide matrices and for all
        // half-precision ones - each worth 1-3 % over 256
        case DL_NB1_WIDE: if (f32) launch_dl<WT, 1, 4, 1, false, 512>(a, sb, st); else launch_dl<WT, 1, 8, 1, false, 512>(a, sb, st); break;
        case DL_NB1_LONGK: if (f32) launch_dl<WT, 1, 4, 2, true>(a, sb, st); else launch_dl<WT, 1, 4, 1, false, 512>(a, sb, st); break;
        case DL_NB1_SQUARE: if (f32) launch_dl<WT, 1, 2, 4>(a, sb, st); else launch_dl<WT, 1, 4, 1, false, 512>(a, sb, st); break;
        case DL_NB2: launch_dl<WT, 2, 4, 2>(a, sb, st); break;
        case DL_NB4: launch_dl<WT, 4, 4, 2>(a, sb, st); break;
        default: launch_dl<WT, 8, 4, 1>(a, sb, st); break;
    }
}

void launch_decode_linear(const DecodeLinear& a, const SeqBatch& sb, hipStream_t st) {
    if (a.wt == DT_F32) launch_dl_t<float>(a, sb, st);
    else launch_dl_t<f16_t>(a, sb, st);
}

// ---------------------------------------------------------------------------------------
// Linear layer for up to 16 activation rows with half weights: from about 8 rows on (16 FMAs
// per weight element at 16) the vector ALUs could no longer keep up with the HBM stream, so
// the products run on the matrix cores: D[n][b] = sum_k W[n][k] x[b][k] with
// v_mfma_f32_16x16x32_f16, the activation rows filling the MFMA's second dimension (rows past
// the batch are zero).
// A workgroup owns 16 * TILES consecutive rows of W; its WAVES waves split K in interleaved
// 64-element blocks, U of them in flight per wave, and meet in LDS (fixed order).  Lane
// (row = lane%16, g = lane/16) supplies elements 32*j + 8*g + (0..7) of a block to MFMA j on
// both operands, so every load instruction reads 64 contiguous bytes per row.  Activations
// arrive rounded to half; with norm_xb they are the un-normalised residual stream, and the
// RMSNorm row scale (gains folded into W) comes from the fragments loaded for the MFMAs.
// ---------------------------------------------------------------------------------------
typedef _Float16 f16x8_d __attribute__((ext_vector_type(8)));
typedef float f32x4_d __attribute__((ext_vector_type(4)));

// What the epilogue of the matrix-core projection kernels reads from memory, fetched by each
// thread for its own outputs BEFORE the weight stream starts (element id = tid + i * THREADS of
// the workgroup's [rows][16] outputs, pair id likewise of its [row pairs][16]): the end of the
// workgroup is then arithmetic and stores, not a chain of dependent loads that every workgroup
// of the launch would sit in at the same time.
template <int TILES, int WAVES>
struct MfmaEpiloguePre {
    static constexpr int ROWS = 16 * TILES, THREADS = 64 * WAVES;
    static constexpr int NS = (ROWS * 16 + THREADS - 1) / THREADS;   // single outputs per thread
    static constexpr int NP = (ROWS * 8 + THREADS - 1) / THREADS;    // output pairs per thread
    float resid[NS];
    float2 cs[NP];
    size_t at[NP];
};

template <int TILES, int WAVES>
__device__ __forceinline__ void mfma_epilogue_prefetch(const DecodeLinear& a, const SeqBatch& sb, int row0, int row_end,
                                                       MfmaEpiloguePre<TILES, WAVES>& p) {
    typedef MfmaEpiloguePre<TILES, WAVES> P;
    const int tid = threadIdx.x;
    if (a.epi == EPI_RESID) {
#pragma unroll
        for (int i = 0; i < P::NS; ++i) {
            const int id = tid + i * P::THREADS, r = id >> 4, b = id & 15, n = row0 + r;
            p.resid[i] = (id < P::ROWS * 16 && n < row_end && b < a.nb) ? a.resid[static_cast<size_t>(b) * a.N + n] : 0.f;
        }
    } else if (a.epi == EPI_QKV) {
        const int dh = a.kv.dh, nq = a.hq * dh, nk = a.kv.hkv * dh;
#pragma unroll
        for (int i = 0; i < P::NP; ++i) {
            const int id = tid + i * P::THREADS, j = id >> 4, b = id & 15, n0 = row0 + 2 * j;
            p.cs[i] = make_float2(1.f, 0.f);
            p.at[i] = 0;
            if (id < P::ROWS * 8 && n0 < row_end && b < a.nb) {
                const int pos = sb.pos[b], e = n0 % dh;
                if (n0 < nq + nk) p.cs[i] = a.rope[static_cast<size_t>(pos) * (dh / 2) + e / 2];
                if (n0 >= nq) {
                    const int hk = (n0 - nq - (n0 < nq + nk ? 0 : nk)) / dh;
                    p.at[i] = kv_row_div(a.kv, a.kv.block_table + static_cast<size_t>(sb.seq[b]) * a.kv.max_pages, pos, hk) * dh + e;
                }
            }
        }
    }
}

// Tail shared by the matrix-core projection kernels: the waves' partial accumulators (and sums
// of squares) meet in LDS, every output is summed over the waves in fixed order by the thread
// that stores it, then the epilogue.  s_red [WAVES][16 TILES][16] and s_ssq [WAVES][16] are LDS
// scratch of the caller.
template <int TILES, int WAVES>
__device__ __forceinline__ void mfma_linear_finish(const DecodeLinear& a, const f32x4_d (&acc)[TILES], float ssq,
                                                   int row0, int row_end, float* s_red, float* s_ssq,
                                                   const MfmaEpiloguePre<TILES, WAVES>& pre) {
    typedef MfmaEpiloguePre<TILES, WAVES> P;
    constexpr int ROWS = 16 * TILES;
    constexpr int THREADS = 64 * WAVES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int K = a.K;
    // D[n][b]: register v of a lane is row 4*g + v of its tile, activation row l16
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) s_red[(wave * ROWS + t * 16 + g * 4 + v) * 16 + l16] = acc[t][v];
    ssq += __shfl_xor(ssq, 16, 64);   // the four lanes of an activation row hold different k
    ssq += __shfl_xor(ssq, 32, 64);
    if (g == 0) s_ssq[wave * 16 + l16] = ssq;
    __syncthreads();
    auto total = [&](int r, int b) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += s_red[(w * ROWS + r) * 16 + b];
        if (a.norm_xb) {
            float q = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) q += s_ssq[w * 16 + b];
            v *= 1.0f / sqrtf(q / static_cast<float>(K) + a.eps);
        }
        return v;
    };

    if (a.epi == EPI_RESID) {
#pragma unroll
        for (int i = 0; i < P::NS; ++i) {
            const int id = tid + i * THREADS, r = id >> 4, b = id & 15, n = row0 + r;
            if (id < ROWS * 16 && n < row_end && b < a.nb) {
                const size_t at = static_cast<size_t>(b) * a.N + n;
                const float y = pre.resid[i] + total(r, b);
                a.out[at] = y;
                if (a.out_h) static_cast<f16_t*>(a.out_h)[at] = store_cast<f16_t>(y, a.oflow);
            }
        }
        return;
    }
    // pair epilogues: one (row pair j, activation row b) per thread and trip
    const int dh = a.kv.dh, nq = a.hq * dh, nk = a.kv.hkv * dh;
#pragma unroll
    for (int i = 0; i < P::NP; ++i) {   // ROWS/2 row pairs x 16 activation rows
        const int id = tid + i * THREADS, j = id >> 4, b = id & 15;
        const int n0 = row0 + 2 * j;
        if (id >= ROWS * 8 || n0 >= row_end || b >= a.nb) continue;
        const float v0 = total(2 * j, b), v1 = total(2 * j + 1, b);
        if (a.epi == EPI_SWIGLU) {
            const int F = a.N / 2;
            static_cast<f16_t*>(a.out_b)[static_cast<size_t>(b) * F + n0 / 2] = store_cast<f16_t>(v0 / (1.0f + expf(-v0)) * v1, a.oflow);
            continue;
        }
        if (n0 < nq + nk) {
            const float2 cs = pre.cs[i];
            const float r0 = v0 * cs.x - v1 * cs.y, r1 = v0 * cs.y + v1 * cs.x;
            if (n0 < nq) {
                a.q[static_cast<size_t>(b) * nq + n0] = r0;
                a.q[static_cast<size_t>(b) * nq + n0 + 1] = r1;
                continue;
            }
            f16_t* kp = static_cast<f16_t*>(a.kv.k);
            kp[pre.at[i]] = store_cast<f16_t>(r0, a.oflow);
            kp[pre.at[i] + 1] = store_cast<f16_t>(r1, a.oflow);
            continue;
        }
        f16_t* vp = static_cast<f16_t*>(a.kv.v);
        vp[pre.at[i]] = store_cast<f16_t>(v0, a.oflow);
        vp[pre.at[i] + 1] = store_cast<f16_t>(v1, a.oflow);
    }
}


template <int TILES, int U, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void decode_linear_mfma_kernel(DecodeLinear a, SeqBatch sb, int rows_wg) {
    constexpr int ROWS = 16 * TILES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    // rows_wg <= ROWS rows per workgroup (even): the launch picks it so that the workgroups
    // come out as a whole number of rounds over the compute units
    const int row0 = blockIdx.x * rows_wg;
    const int row_end = min(row0 + rows_wg, a.N);
    const f16_t* __restrict__ W = static_cast<const f16_t*>(a.W);
    const f16_t* __restrict__ X = static_cast<const f16_t*>(a.xb);
    const int K = a.K, nblk = K / 64;  // K is a multiple of 64 on this path
    // Every workgroup walks K from its own starting block.  Workgroups of one launch run in
    // lockstep, and with rows a power of two apart they would all ask the same few memory
    // channels for the same k offset at the same time (measured: 4.8 -> 6.1 TB/s at K = 8192).
    const int rot = static_cast<int>((blockIdx.x * 37u) % static_cast<unsigned>(nblk));

    const f16_t* wp[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t)   // lanes past the workgroup's rows re-read its last row (a cache hit; never stored)
        wp[t] = W + static_cast<size_t>(min(row0 + t * 16 + l16, row_end - 1)) * K + g * 8;
    const f16_t* xp = X + static_cast<size_t>(l16 < a.nb ? l16 : 0) * K + g * 8;

    MfmaEpiloguePre<TILES, WAVES> pre;
    mfma_epilogue_prefetch<TILES, WAVES>(a, sb, row0, row_end, pre);

    f32x4_d acc[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[t][v] = 0.f;
    float ssq = 0.f;

    for (int kb0 = wave; kb0 < nblk; kb0 += WAVES * U) {
        uint4 wv[U][TILES][2], xv[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kb = kb0 + WAVES * u;
            int kc = (kb < nblk ? kb : kb0) + rot;  // past the end: re-read a valid block, zero its activations
            if (kc >= nblk) kc -= nblk;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int t = 0; t < TILES; ++t) wv[u][t][j] = *reinterpret_cast<const uint4*>(wp[t] + kc * 64 + j * 32);
                xv[u][j] = kb < nblk ? *reinterpret_cast<const uint4*>(xp + kc * 64 + j * 32) : make_uint4(0u, 0u, 0u, 0u);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (a.norm_xb) {  // sum of squares of this lane's activation row, for the RMSNorm scale
                    const f16x8_d h = __builtin_bit_cast(f16x8_d, xv[u][j]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) ssq = fmaf(static_cast<float>(h[e]), static_cast<float>(h[e]), ssq);
                }
#pragma unroll
                for (int t = 0; t < TILES; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_d, wv[u][t][j]),
                                                                    __builtin_bit_cast(f16x8_d, xv[u][j]), acc[t], 0, 0, 0);
            }
    }

    __shared__ float s_red[WAVES * ROWS * 16];
    __shared__ float s_ssq[WAVES * 16];
    mfma_linear_finish<TILES, WAVES>(a, acc, ssq, row0, row_end, s_red, s_ssq, pre);
}

// ---------------------------------------------------------------------------------------
// The same projection with the weights streamed through LDS by direct loads, for workgroups
// of at most 64 rows (projections back to d_model: 32 rows per workgroup at the 70B width).
// The register kernel above keeps (TILES + 1) x 16 bytes per lane in flight, about 50 KB per
// compute unit at 32 rows, and reads 64-byte pieces of 16 rows per instruction; here a ring of
// STAGES k-steps of 256 elements (512 contiguous bytes per row and load instruction) holds up
// to 120 KB of loads in flight per compute unit and costs no registers.  Eight waves; per
// k-step wave w multiplies elements 32 w .. 32 w + 31: one 16-byte LDS read per row tile
// plus one for the activations (16-byte chunks XOR-swizzled by row, the swizzle applied on the
// global side), TILES MFMAs, one barrier.  K must be a multiple of 256.
// ---------------------------------------------------------------------------------------
template <int TILES, int STAGES>
__global__ __launch_bounds__(512) void decode_linear_dma_kernel(DecodeLinear a, SeqBatch sb, int rows_wg) {
    constexpr int WAVES = 8, ROWS = 16 * TILES, BK = 256, ROWB = BK * 2;
    constexpr int STAGE_B = (ROWS + 16) * ROWB;          // weight rows, then the 16 activation rows
    constexpr int NLOAD = (ROWS + 16) / 2;               // wave-level loads per stage: two rows each
    constexpr int NPER = NLOAD / WAVES;
    static_assert(NLOAD % WAVES == 0, "loads must divide evenly over the waves");
    static_assert(NPER * (STAGES - 1) < 64, "vmcnt is a 6-bit counter");
    static_assert(STAGES * STAGE_B >= (WAVES * ROWS * 16 + ROWS * 16 + WAVES * 16) * 4, "the reduction reuses the ring");
    extern __shared__ __attribute__((aligned(16))) char smem_dl[];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)smem_dl));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int row0 = blockIdx.x * rows_wg;
    const int row_end = min(row0 + rows_wg, a.N);
    const f16_t* __restrict__ W = static_cast<const f16_t*>(a.W);
    const f16_t* __restrict__ X = static_cast<const f16_t*>(a.xb);
    const int K = a.K, ksteps = K / BK;
    const int rot = static_cast<int>((blockIdx.x * 37u) % static_cast<unsigned>(ksteps));   // see the register kernel

    const f16_t* src[NPER];
    uint32_t dst[NPER];
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
        const int c = wave + WAVES * i;                  // this wave's i-th load of a stage: stage rows 2c, 2c + 1
        const int r = 2 * c + (lane >> 5), slot = lane & 31;
        const bool is_w = r < ROWS;
        const int rr = is_w ? r : r - ROWS;              // row within its tile block: the swizzle key
        const int chunk = slot ^ (rr & 31);
        // rows past the workgroup's share re-read its last row, activation rows past the batch row 0:
        // both feed accumulators that are never stored
        const int grow = is_w ? min(row0 + r, row_end - 1) : (rr < a.nb ? rr : 0);
        src[i] = (is_w ? W : X) + static_cast<size_t>(grow) * K + chunk * 8;
        dst[i] = lds0 + c * 1024;
    }
    auto issue = [&](int ks) {                           // k-step ks -> stage ks % STAGES
        int kc = (ks < ksteps ? ks : ksteps - 1) + rot;  // past the end: a harmless reload into a free stage
        if (kc >= ksteps) kc -= ksteps;
        const uint32_t sb0 = static_cast<uint32_t>(ks % STAGES) * STAGE_B;
#pragma unroll
        for (int i = 0; i < NPER; ++i) lds_dma16(src[i] + static_cast<size_t>(kc) * BK, dst[i] + sb0);
    };

    f32x4_d acc[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) acc[t] = f32x4_d{0.f, 0.f, 0.f, 0.f};
    float ssq = 0.f;

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s);
    MfmaEpiloguePre<TILES, WAVES> pre;               // after the first stages are on their way
    mfma_epilogue_prefetch<TILES, WAVES>(a, sb, row0, row_end, pre);
    for (int ks = 0; ks < ksteps; ++ks) {
        wait_vmcnt<NPER*(STAGES - 2)>();                 // this wave's loads of step ks have landed
        __syncthreads();                                 // ... everyone's; and stage (ks-1) % STAGES is free
        const char* sW = smem_dl + (ks % STAGES) * STAGE_B;
        const char* sX = sW + ROWS * ROWB;
        const int cw = 4 * wave + g;                     // this lane's 16-byte chunk of the step
        const uint4 xf = *reinterpret_cast<const uint4*>(sX + l16 * ROWB + ((cw ^ l16) << 4));
        uint4 wf[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int r = t * 16 + l16;
            wf[t] = *reinterpret_cast<const uint4*>(sW + r * ROWB + ((cw ^ (r & 31)) << 4));
        }
        issue(ks + STAGES - 1);                          // issued under the latency of the LDS reads
        if (a.norm_xb) {
            const f16x8_d h = __builtin_bit_cast(f16x8_d, xf);
#pragma unroll
            for (int e = 0; e < 8; ++e) ssq = fmaf(static_cast<float>(h[e]), static_cast<float>(h[e]), ssq);
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_d, wf[t]), __builtin_bit_cast(f16x8_d, xf),
                                                            acc[t], 0, 0, 0);
    }
    wait_vmcnt<0>();                                     // the reloads past the end
    __syncthreads();                                     // the ring is free: it becomes the reduction's scratch
    float* s_red = reinterpret_cast<float*>(smem_dl);
    float* s_ssq = s_red + WAVES * ROWS * 16;
    mfma_linear_finish<TILES, WAVES>(a, acc, ssq, row0, row_end, s_red, s_ssq, pre);
}

template <int TILES, int STAGES>
static void launch_dl_dma(const DecodeLinear& a, const SeqBatch& sb, dim3 grid, int rows, hipStream_t st) {
    constexpr size_t lds = static_cast<size_t>(STAGES) * (16 * TILES + 16) * 512;
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    static std::once_flag once;  // more than 64 KB of LDS per workgroup is an opt-in
    std::call_once(once, [] {
        note_kernel_attribute(hipFuncSetAttribute(reinterpret_cast<const void*>(decode_linear_dma_kernel<TILES, STAGES>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    });
    launch((decode_linear_dma_kernel<TILES, STAGES>), grid, dim3(512), lds, st, a, sb, rows);
}

// Variant and rows per workgroup of the matrix-core projection for an [N, K] matrix: ids 0..3 are
// the LDS-ring kernel with 1..4 row tiles, ids 4..11 the register kernel with 1..8 row tiles.
static const char* const DLM_NAMES[12] = {
    "f16 mfma lds-ring 1 tile", "f16 mfma lds-ring 2 tiles", "f16 mfma lds-ring 3 tiles", "f16 mfma lds-ring 4 tiles",
    "f16 mfma reg 1 tile", "f16 mfma reg 2 tiles", "f16 mfma reg 3 tiles", "f16 mfma reg 4 tiles",
    "f16 mfma reg 5 tiles", "f16 mfma reg 6 tiles", "f16 mfma reg 7 tiles", "f16 mfma reg 8 tiles"};
const char* decode_linear_mfma_variant_name(int id) { return id >= 0 && id < 12 ? DLM_NAMES[id] : nullptr; }

int choose_decode_linear_mfma(int N, int K, int* rows_wg) {
    // Rows per workgroup: the workgroups of a launch should come out as whole rounds over the
    // 256 compute units (a launch of 160 or 448 workgroups leaves units idle for a good part of
    // it: 70B-shape QKV 44 -> 31 us), with as many rows per workgroup as fit (each activation
    // fragment then feeds more row tiles), up to 128.
    constexpr int CUS = 256;
    const int rounds = ((N + CUS - 1) / CUS + 127) / 128;
    int rows = (N + CUS * rounds - 1) / (CUS * rounds);
    rows += rows & 1;   // the pair epilogues need even row offsets
    if (rows < 16) rows = 16;
    *rows_wg = rows;
    const int tiles = (rows + 15) / 16;
    // Weights through an LDS ring of direct loads - unless the row pitch is a power of two: then
    // the rows of a workgroup sit in the same few memory channels, and a workgroup that moves in
    // lockstep from barrier to barrier asks them all at once (70B QKV, K = 8192: 31 -> 44 us, while
    // K = 28672, 13824, 11008 and 5120 gain 9..20 %); the register kernel's waves drift apart.
    if (rows <= 64 && K % 256 == 0 && K / 256 >= 8 && (K & (K - 1)) != 0) return tiles - 1;
    return 4 + tiles - 1;
}

void launch_decode_linear_mfma(const DecodeLinear& a, const SeqBatch& sb, hipStream_t st) {
    int rows = 0;
    const int id = choose_decode_linear_mfma(a.N, a.K, &rows);
    const dim3 grid((a.N + rows - 1) / rows);
    switch (id) {
        case 0: launch_dl_dma<1, 8>(a, sb, grid, rows, st); break;
        case 1: launch_dl_dma<2, 6>(a, sb, grid, rows, st); break;
        case 2: launch_dl_dma<3, 4>(a, sb, grid, rows, st); break;
        case 3: launch_dl_dma<4, 3>(a, sb, grid, rows, st); break;
        // one K block in flight per wave; 8 waves split K, 16 for tall workgroups
        case 4: launch((decode_linear_mfma_kernel<1, 1, 8>), grid, dim3(512), 0, st, a, sb, rows); break;
        case 5: launch((decode_linear_mfma_kernel<2, 1, 8>), grid, dim3(512), 0, st, a, sb, rows); break;
        case 6: launch((decode_linear_mfma_kernel<3, 1, 8>), grid, dim3(512), 0, st, a, sb, rows); break;
        case 7: launch((decode_linear_mfma_kernel<4, 1, 8>), grid, dim3(512), 0, st, a, sb, rows); break;
        case 8: launch((decode_linear_mfma_kernel<5, 1, 16>), grid, dim3(1024), 0, st, a, sb, rows); break;
        case 9: launch((decode_linear_mfma_kernel<6, 1, 16>), grid, dim3(1024), 0, st, a, sb, rows); break;
        case 10: launch((decode_linear_mfma_kernel<7, 1, 16>), grid, dim3(1024), 0, st, a, sb, rows); break;
        default: launch((decode_linear_mfma_kernel<8, 1, 16>), grid, dim3(1024), 0, st, a, sb, rows); break;
    }
}

// ---------------------------------------------------------------------------------------
// Attention of one new token per sequence over its cached keys/values.
// Grid (nsplit, nb*hq).  A workgroup takes one slice of the context of one (sequence,
// query head); TPT = DH/VEC adjacent lanes share a token (one 16-byte load each), and each
// lane group keeps TU tokens in flight, so a workgroup covers TU*256/TPT tokens per trip.
// Each lane group keeps its own running (max, sum, weighted V) - softmax statistics are
// merged with lane shuffles inside the group and through LDS across groups; the slices
// of one (sequence, head) are merged by decode_attn_merge_kernel in slice order (a second
// launch: a device-wide fence per workgroup costs far more than a kernel boundary).
// ---------------------------------------------------------------------------------------
constexpr int ATTN_MAX_SPLIT = 32;

template <typename KT, int DH, int TU, int GQ>
__global__ __launch_bounds__(256) void decode_attn_kernel(DecodeAttn a, SeqBatch sb) {
    constexpr int VEC = Elem<KT>::VEC;
    constexpr int TPT = DH / VEC;
    constexpr int GROUPS = 256 / TPT;
    const int tid = threadIdx.x;
    const int split = blockIdx.x;
    const int hgroups = a.hq / GQ;                 // GQ consecutive query heads (one KV head) per workgroup
    const int b = blockIdx.y / hgroups, h0 = (blockIdx.y % hgroups) * GQ;
    const int hk = h0 / (a.hq / a.kv.hkv);
    const int seq = sb.seq[b];
    const int ctx = sb.pos[b] + 1;  // the new token's k,v are already in the cache
    const int per = (ctx + a.nsplit - 1) / a.nsplit;
    const int u_begin = split * per, u_end = min(ctx, u_begin + per);
    const int g = tid / TPT, e0 = (tid % TPT) * VEC;
    const float scale = 1.0f / sqrtf(static_cast<float>(DH));
    const KT* __restrict__ kp = static_cast<const KT*>(a.kv.k);
    const KT* __restrict__ vp = static_cast<const KT*>(a.kv.v);
    const int32_t* bt = a.kv.block_table + static_cast<size_t>(seq) * a.kv.max_pages;

    float qv[GQ][VEC];
#pragma unroll
    for (int q = 0; q < GQ; ++q) {
        const float* qp = a.q + static_cast<size_t>(b) * a.hq * DH + (h0 + q) * DH + e0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) qv[q][e] = qp[e] * scale;
    }
    float m[GQ], l[GQ], acc[GQ][VEC];
#pragma unroll
    for (int q = 0; q < GQ; ++q) {
        m[q] = -INFINITY;
        l[q] = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[q][e] = 0.f;
    }

    // The slice's block-table entries go to LDS once, so that a trip's K/V addresses need no
    // global load of their own; a slice with more pages than fit looks them up in memory.
    constexpr int PG_CAP = 512;
    __shared__ int32_t s_pg[PG_CAP];
    const int pg_lo = u_begin < u_end ? u_begin / a.kv.page : 0;
    const int pg_n = u_begin < u_end ? (u_end - 1) / a.kv.page - pg_lo + 1 : 0;
    const bool pg_cached = pg_n <= PG_CAP;
    if (pg_cached)
        for (int i = tid; i < pg_n; i += 256) s_pg[i] = bt[pg_lo + i];
    __syncthreads();

    // One trip = TU tokens per lane group; the loads of trip t+1 are issued before trip t is
    // worked on (the kernel is latency-bound: few trips, each a dependent chain of loads).
    uint4 ka[TU], va[TU], kb[TU], vb[TU];          // two register sets, used alternately
    auto fetch = [&](int u0, uint4 (&kr)[TU], uint4 (&vr)[TU]) {
#pragma unroll
        for (int i = 0; i < TU; ++i) {
            const int u = u0 + i * GROUPS;
            const int uc = u < u_end ? u : u_end - 1;
            const int pg = uc / a.kv.page, slot = uc - pg * a.kv.page;
            const int page_id = pg_cached ? s_pg[pg - pg_lo] : bt[pg];
            const size_t at = ((static_cast<size_t>(page_id) * a.kv.hkv + hk) * a.kv.page + slot) * DH + e0;
            kr[i] = *reinterpret_cast<const uint4*>(kp + at);
            vr[i] = *reinterpret_cast<const uint4*>(vp + at);
        }
    };
    auto widen = [](const uint4& r, float* out) {
        if constexpr (sizeof(KT) == 4) {
            out[0] = __uint_as_float(r.x); out[1] = __uint_as_float(r.y);
            out[2] = __uint_as_float(r.z); out[3] = __uint_as_float(r.w);
        } else {
            typedef _Float16 h8 __attribute__((ext_vector_type(8)));
            const h8 t = __builtin_bit_cast(h8, r);
#pragma unroll
            for (int e = 0; e < 8; ++e) out[e] = static_cast<float>(t[e]);
        }
    };
    auto work = [&](int u0, const uint4 (&kr)[TU], const uint4 (&vr)[TU]) {
        float kf[TU][VEC], vf[TU][VEC];
        bool ok[TU];
#pragma unroll
        for (int i = 0; i < TU; ++i) {
            ok[i] = u0 + i * GROUPS < u_end;
            widen(kr[i], kf[i]);
            widen(vr[i], vf[i]);
        }
#pragma unroll
        for (int q = 0; q < GQ; ++q) {
            float s[TU], mn = m[q];
#pragma unroll
            for (int i = 0; i < TU; ++i) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) d = fmaf(qv[q][e], kf[i][e], d);
                d = group_sum<TPT>(d);
                s[i] = ok[i] ? d : -INFINITY;
                mn = fmaxf(mn, s[i]);
            }
            const float corr = __expf(m[q] - mn);  // first trip: exp(-inf) = 0
            l[q] *= corr;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[q][e] *= corr;
#pragma unroll
            for (int i = 0; i < TU; ++i) {
                const float p = __expf(s[i] - mn);
                l[q] += p;
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[q][e] = fmaf(p, vf[i][e], acc[q][e]);
            }
            m[q] = mn;
        }
    };
    constexpr int STEP = GROUPS * TU;
    int u0 = u_begin + g;
    if (u0 < u_end) fetch(u0, ka, va);
    while (u0 < u_end) {
        if (u0 + STEP < u_end) fetch(u0 + STEP, kb, vb);
        work(u0, ka, va);
        u0 += STEP;
        if (u0 >= u_end) break;
        if (u0 + STEP < u_end) fetch(u0 + STEP, ka, va);
        work(u0, kb, vb);
        u0 += STEP;
    }

    __shared__ float s_m[GQ][GROUPS], s_l[GQ][GROUPS];
    __shared__ float s_acc[GQ][GROUPS][DH];
#pragma unroll
    for (int q = 0; q < GQ; ++q) {
        if (tid % TPT == 0) { s_m[q][g] = m[q]; s_l[q][g] = l[q]; }
#pragma unroll
        for (int e = 0; e < VEC; ++e) s_acc[q][g][e0 + e] = acc[q][e];
    }
    __syncthreads();

    if (tid >= DH) return;
#pragma unroll
    for (int q = 0; q < GQ; ++q) {
        float M = -INFINITY, L = 0.f, O = 0.f;
#pragma unroll
        for (int i = 0; i < GROUPS; ++i) M = fmaxf(M, s_m[q][i]);
        if (M > -INFINITY) {
#pragma unroll
            for (int i = 0; i < GROUPS; ++i) {
                const float w = __expf(s_m[q][i] - M);  // empty groups: exp(-inf) = 0
                L = fmaf(s_l[q][i], w, L);
                O = fmaf(s_acc[q][i][tid], w, O);
            }
        }
        const int bh = b * a.hq + h0 + q;
        if (a.nsplit == 1) {
            const size_t at = static_cast<size_t>(bh) * DH + tid;
            if (a.o_dtype == DT_F32) static_cast<float*>(a.o)[at] = O / L;
            else static_cast<f16_t*>(a.o)[at] = static_cast<f16_t>(O / L);
            continue;
        }
        const size_t pbase = static_cast<size_t>(bh) * a.nsplit;
        a.part_o[(pbase + split) * DH + tid] = O;
        if (tid == 0) {
            a.part_ml[(pbase + split) * 2] = M;
            a.part_ml[(pbase + split) * 2 + 1] = L;
        }
    }
}

// Merge of the context slices of one (sequence, head): grid nb*hq, DH threads.  Lanes
// 0..31 fetch the slice statistics in parallel; the weighted sum runs in slice order.
template <int DH>
__global__ __launch_bounds__(DH) void decode_attn_merge_kernel(DecodeAttn a) {
    const int tid = threadIdx.x, bh = blockIdx.x;
    const size_t pbase = static_cast<size_t>(bh) * a.nsplit;
    __shared__ float s_w[ATTN_MAX_SPLIT];
    __shared__ float s_L;
    // the partial outputs do not depend on the slice weights: their loads go out first and are in
    // flight while the weights are worked out (one memory round trip instead of two in a row)
    float po[ATTN_MAX_SPLIT];
#pragma unroll
    for (int s = 0; s < ATTN_MAX_SPLIT; ++s) po[s] = s < a.nsplit ? a.part_o[(pbase + s) * DH + tid] : 0.f;
    if (tid < ATTN_MAX_SPLIT) {
        const bool have = tid < a.nsplit;
        const float ms = have ? a.part_ml[(pbase + tid) * 2] : -INFINITY;
        const float ls = have ? a.part_ml[(pbase + tid) * 2 + 1] : 0.f;
        float mx = ms;
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        const float w = ms == -INFINITY ? 0.f : __expf(ms - mx);  // slices without tokens weigh 0
        float lw = ls * w;
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) lw += __shfl_xor(lw, o, 64);
        s_w[tid] = w;
        if (tid == 0) s_L = lw;
    }
    __syncthreads();
    float ox = 0.f;
#pragma unroll
    for (int s = 0; s < ATTN_MAX_SPLIT; ++s) ox = fmaf(po[s], s_w[s], ox);
    const size_t at = static_cast<size_t>(bh) * DH + tid;
    if (a.o_dtype == DT_F32) static_cast<float*>(a.o)[at] = ox / s_L;
    else static_cast<f16_t*>(a.o)[at] = static_cast<f16_t>(ox / s_L);
}

// ---------------------------------------------------------------------------------------
// Grouped-query variant for half caches with dh = 128 and 4..16 query heads per KV head
// (the 70B shape: 8).  The vector-ALU kernel above is bound by its FMAs and lane reductions
// once several heads share every key; here both products run on the matrix cores, with the
// heads of one KV head as the 16-wide dimension and a tile of 16 tokens per wave and trip:
//   S^T[token][head] = K[token][:] . q[head][:]   4 x v_mfma_f32_16x16x32_f16; lane (token,
//       g) loads 16 bytes of its key row at dh offset 32 j + 8 g straight from the cache;
//   O[head][dh] += P[head][token] V[token][dh]    8 x v_mfma_f32_16x16x16_f16; the S^T
//       accumulators (lane (head, g): tokens 4g..4g+3) are, after exp, exactly the A
//       operand; V rows go through a 4 KB LDS tile per wave (same addresses as K) and come
//       back transposed by ds_read_b64_tr_b16 as the B operand.
// Grid (nsplit, nb * hkv); the waves of a workgroup take tiles in turn and meet in LDS.  Every
// workgroup pays a fixed chain of dependent steps (block table, q, first tile, merge: about
// 8 us) and sliced contexts a merge launch on top, so up to 1024 tokens one workgroup of 8
// waves takes the whole context of its (sequence, KV head) (16 x 8 units, 576 tokens: 13.4 us
// against 12.0 + 4.1 us for four slices and their merge; 16 waves: 15.0 us); longer contexts are
// cut into slices for 4-wave workgroups and merged by decode_attn_merge_kernel as above.
// ---------------------------------------------------------------------------------------
typedef _Float16 f16x4_d __attribute__((ext_vector_type(4)));

template <int WAVES, bool TWOSETS>   // TWOSETS: the next tile's K/V are loaded while the current one is worked on
__global__ __launch_bounds__(64 * WAVES) void decode_attn_gqa_kernel(DecodeAttn a, SeqBatch sb) {
    constexpr int DH = 128, KJ = DH / 32, NT = DH / 16, GH = 16, THREADS = 64 * WAVES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, g = lane >> 4;
    const int G = a.hq / a.kv.hkv;
    const int split = blockIdx.x, b = blockIdx.y / a.kv.hkv, hk = blockIdx.y % a.kv.hkv;
    const int h0 = hk * G;
    const int seq = sb.seq[b];
    const int ctx = sb.pos[b] + 1;  // the new token's k,v are already in the cache
    const int per = (ctx + a.nsplit - 1) / a.nsplit;
    const int u_begin = split * per, u_end = min(ctx, u_begin + per);
    const f16_t* __restrict__ kp = static_cast<const f16_t*>(a.kv.k);
    const f16_t* __restrict__ vp = static_cast<const f16_t*>(a.kv.v);
    const int32_t* bt = a.kv.block_table + static_cast<size_t>(seq) * a.kv.max_pages;

    // q of head l16 (heads past G are zero): loaded first, so that the loads overlap the block-table
    // round trip below; scaled by 1/sqrt(dh) in fp32 and rounded to half once
    float4 qraw[KJ][2];
    {
        const float* qp = a.q + (static_cast<size_t>(b) * a.hq + h0 + (l16 < G ? l16 : 0)) * DH + 8 * g;
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
            qraw[j][0] = *reinterpret_cast<const float4*>(qp + 32 * j);
            qraw[j][1] = *reinterpret_cast<const float4*>(qp + 32 * j + 4);
        }
    }

    typedef uint32_t u32x4_d __attribute__((ext_vector_type(4)));
    u32x4_d ka[KJ], kb[KJ], va[KJ], vb[KJ];   // two register sets, used alternately
    constexpr int PG_CAP = 512;
    __shared__ int32_t s_pg[PG_CAP];
    const int pg_lo = u_begin < u_end ? u_begin / a.kv.page : 0;
    const int pg_n = u_begin < u_end ? (u_end - 1) / a.kv.page - pg_lo + 1 : 0;
    const bool pg_cached = pg_n <= PG_CAP;
    auto fetch = [&](int t0, u32x4_d (&kr)[KJ], u32x4_d (&vr)[KJ], bool staged) {
        const int u = min(t0 + l16, u_end - 1);   // past the slice: re-read its last token, masked below
        const int pg = u / a.kv.page, slot = u - pg * a.kv.page;
        const int page_id = staged ? s_pg[pg - pg_lo] : bt[pg];
        const size_t at = ((static_cast<size_t>(page_id) * a.kv.hkv + hk) * a.kv.page + slot) * DH + 8 * g;
#pragma unroll
        for (int j = 0; j < KJ; ++j) kr[j] = *reinterpret_cast<const u32x4_d*>(kp + at + 32 * j);
#pragma unroll
        for (int j = 0; j < KJ; ++j) vr[j] = *reinterpret_cast<const u32x4_d*>(vp + at + 32 * j);
    };
    constexpr int STEP = 16 * WAVES;
    int t0 = u_begin + 16 * wave;
    // the slice's page ids go to LDS once (reading the first tile's ids straight from the block
    // table instead, ahead of the barrier, measured no faster)
    if (pg_cached)
        for (int i = tid; i < pg_n; i += THREADS) s_pg[i] = bt[pg_lo + i];
    __syncthreads();
    if (t0 < u_end) fetch(t0, ka, va, pg_cached);

    f16x8_d qf[KJ];
    {
        const float scale = l16 < G ? 1.0f / sqrtf(static_cast<float>(DH)) : 0.f;
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
            const float t[8] = {qraw[j][0].x, qraw[j][0].y, qraw[j][0].z, qraw[j][0].w,
                                qraw[j][1].x, qraw[j][1].y, qraw[j][1].z, qraw[j][1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[j][e] = static_cast<f16_t>(t[e] * scale);
        }
    }

    float m = -INFINITY, lsum = 0.f;   // of head l16 (lsum: this lane's tokens only until the end)
    f32x4_d o[NT];                     // O[head 4g + v][dh 16 nt + l16]
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) o[nt] = f32x4_d{0.f, 0.f, 0.f, 0.f};
    // one 4 KB V tile [token][dh] per wave (16-byte chunks XOR-swizzled by token); after the
    // token loop the same memory holds the waves' outputs for 8 heads at a time
    __shared__ __align__(16) char s_buf[WAVES * 16 * DH * 2];
    static_assert(WAVES * 16 * DH * 2 >= WAVES * 8 * DH * 4, "output merge fits the V tiles");
    __shared__ __align__(16) float s_c[WAVES][GH];           // rescale factor of the running sums per head

    auto work = [&](int t0, const u32x4_d (&kr)[KJ], const u32x4_d (&vr)[KJ]) {
        char* sv = s_buf + wave * (16 * DH * 2);
#pragma unroll
        for (int j = 0; j < KJ; ++j)   // token row l16, chunk 4 j + g
            *reinterpret_cast<u32x4_d*>(sv + l16 * (DH * 2) + (((4 * j + g) ^ l16) << 4)) = vr[j];
        f32x4_d acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KJ; ++j)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_d, kr[j]), qf[j], acc, 0, 0, 0);
        // register v of lane (head l16, g) is token t0 + 4 g + v
        float sc[4], mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            sc[v] = t0 + 4 * g + v < u_end ? acc[v] : -INFINITY;
            mx = fmaxf(mx, sc[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));   // finite: the tile holds at least one token of the slice
        const float mn = fmaxf(m, mx);
        const float corr = __expf(m - mn);        // first tile: exp(-inf) = 0
        float ps = 0.f;
        f16x4_d pf;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float p = __expf(sc[v] - mn);
            ps += p;
            pf[v] = static_cast<f16_t>(p);
        }
        lsum = fmaf(lsum, corr, ps);
        m = mn;
        if (g == 0) s_c[wave][l16] = corr;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the wave reads back what its other lanes wrote
        __builtin_amdgcn_wave_barrier();
        const float4 c = *reinterpret_cast<const float4*>(&s_c[wave][4 * g]);   // heads 4g..4g+3: the rows of o
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            // B operand V[tokens 4g..4g+3][dh 16 nt + l16]: within 16 lanes, lane x hands in
            // the address of 4 halfs and lane (x / 4, x % 4) = (q, e) receives element e of
            // what lanes q, q + 4, q + 8, q + 12 pointed at; so lane x points at token
            // 4 g + x / 4, features 16 nt + 4 (x % 4) .. + 3.
            typedef short i16x4_t __attribute__((ext_vector_type(4)));
            const int r = 4 * g + (l16 >> 2), d = 16 * nt + 4 * (l16 & 3);
            const char* at = sv + r * (DH * 2) + (((d >> 3) ^ r) << 4) + (d & 7) * 2;
            const i16x4_t vt = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4_t*)(at));
            o[nt][0] *= c.x; o[nt][1] *= c.y; o[nt][2] *= c.z; o[nt][3] *= c.w;
            o[nt] = __builtin_amdgcn_mfma_f32_16x16x16f16(pf, __builtin_bit_cast(f16x4_d, vt), o[nt], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the next tile overwrites s_v and s_c
        __builtin_amdgcn_wave_barrier();
    };
    if constexpr (TWOSETS) {
        while (t0 < u_end) {
            if (t0 + STEP < u_end) fetch(t0 + STEP, kb, vb, pg_cached);
            work(t0, ka, va);
            t0 += STEP;
            if (t0 >= u_end) break;
            if (t0 + STEP < u_end) fetch(t0 + STEP, ka, va, pg_cached);
            work(t0, kb, vb);
            t0 += STEP;
        }
    } else {   // many waves per workgroup: they overlap each other's loads
        while (t0 < u_end) {
            work(t0, ka, va);
            t0 += STEP;
            if (t0 < u_end) fetch(t0, ka, va, pg_cached);
        }
    }

    __shared__ float s_m[WAVES][GH], s_l[WAVES][GH];
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (g == 0) { s_m[wave][l16] = m; s_l[wave][l16] = lsum; }
    float* s_o = reinterpret_cast<float*>(s_buf);   // [WAVES][8][DH]
    for (int hb = 0; hb < G; hb += 8) {             // heads hb .. hb+7: rows of lane groups g = hb/4, hb/4 + 1
        __syncthreads();                            // the V tiles (or the previous 8 heads) are done with
        if ((g >> 1) == (hb >> 3)) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) s_o[(wave * 8 + 4 * (g & 1) + v) * DH + 16 * nt + l16] = o[nt][v];
        }
        __syncthreads();
        for (int id = tid; id < 8 * DH; id += THREADS) {
            const int hl = id / DH, h = hb + hl, e = id % DH;
            if (h >= G) break;
            float M = -INFINITY, L = 0.f, O = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) M = fmaxf(M, s_m[w][h]);
            if (M > -INFINITY) {
#pragma unroll
                for (int w = 0; w < WAVES; ++w) {
                    const float wt = __expf(s_m[w][h] - M);  // waves without a tile: exp(-inf) = 0
                    L = fmaf(s_l[w][h], wt, L);
                    O = fmaf(s_o[(w * 8 + hl) * DH + e], wt, O);
                }
            }
            const int bh = b * a.hq + h0 + h;
            if (a.nsplit == 1) {
                const size_t at = static_cast<size_t>(bh) * DH + e;
                if (a.o_dtype == DT_F32) static_cast<float*>(a.o)[at] = O / L;
                else static_cast<f16_t*>(a.o)[at] = static_cast<f16_t>(O / L);
                continue;
            }
            const size_t pbase = static_cast<size_t>(bh) * a.nsplit;
            a.part_o[(pbase + split) * DH + e] = O;
            if (e == 0) {
                a.part_ml[(pbase + split) * 2] = M;
                a.part_ml[(pbase + split) * 2 + 1] = L;
            }
        }
    }
}

// Whether the grouped-query matrix-core kernel takes a shape.
static bool decode_attn_gqa(int kv_dtype, int dh, int hq, int hkv) {
    const int G = hq / hkv;
    return kv_dtype == DT_F16 && dh == 128 && G >= 4 && G <= 16;
}

// Query heads handled per workgroup: consecutive heads that share a KV head read its keys
// and values once (grouped-query attention).
int decode_attn_heads_per_group(int kv_dtype, int dh, int hq, int hkv) {
    const int G = hq / hkv;
    if (decode_attn_gqa(kv_dtype, dh, hq, hkv)) return G;
    return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1);
}

template <typename KT, int DH>
static void launch_da(const DecodeAttn& a, const SeqBatch& sb, hipStream_t st) {
    const int gq = decode_attn_heads_per_group(a.kv_dtype, DH, a.hq, a.kv.hkv);
    const dim3 grid(a.nsplit, a.nb * a.hq / gq), block(256);
    if (decode_attn_gqa(a.kv_dtype, DH, a.hq, a.kv.hkv)) {
        if (a.nsplit == 1) launch((decode_attn_gqa_kernel<8, false>), grid, dim3(512), 0, st, a, sb);
        else launch((decode_attn_gqa_kernel<4, true>), grid, block, 0, st, a, sb);
    } else if (gq == 4) launch((decode_attn_kernel<KT, DH, 4, 4>), grid, block, 0, st, a, sb);
    else if (gq == 2) launch((decode_attn_kernel<KT, DH, 4, 2>), grid, block, 0, st, a, sb);
    else launch((decode_attn_kernel<KT, DH, 4, 1>), grid, block, 0, st, a, sb);
    if (a.nsplit > 1) launch(decode_attn_merge_kernel<DH>, dim3(a.nb * a.hq), dim3(DH), 0, st, a);
}

void launch_decode_attn(const DecodeAttn& a, const SeqBatch& sb, hipStream_t st) {
    const bool f32 = a.kv_dtype == DT_F32;
    switch (a.kv.dh) {
        case 32: if (f32) launch_da<float, 32>(a, sb, st); else launch_da<f16_t, 32>(a, sb, st); break;
        case 64: if (f32) launch_da<float, 64>(a, sb, st); else launch_da<f16_t, 64>(a, sb, st); break;
        default: if (f32) launch_da<float, 128>(a, sb, st); else launch_da<f16_t, 128>(a, sb, st); break;
    }
}

// Workgroups a launch should have: every workgroup pays a fixed chain of dependent steps
// (block table, q, first tiles, merge), so beyond what fills the chip more slices cost time
// (grouped-query kernel at 16 x 8 units, 576 tokens: 3 slices 17.4 us, 6: 18.8, 8: 28.7).
int decode_attn_target_workgroups(int kv_dtype, int dh, int hq, int hkv) {
    return decode_attn_gqa(kv_dtype, dh, hq, hkv) ? 512 : 768;
}

// Longest context the grouped-query kernel takes in one workgroup per (sequence, KV head)
// (0: the shape does not use that kernel).
int decode_attn_single_pass_ctx(int kv_dtype, int dh, int hq, int hkv) {
    return decode_attn_gqa(kv_dtype, dh, hq, hkv) ? 1024 : 0;
}

int decode_attn_tokens_per_trip(int kv_dtype, int dh, int hq, int hkv) {
    if (decode_attn_gqa(kv_dtype, dh, hq, hkv)) return 64;   // 4 waves x one 16-token tile
    const int vec = kv_dtype == DT_F32 ? 4 : 8;
    return 4 * 256 / (dh / vec);
}

// W[n][k] *= gain[k] on a half matrix, 8 elements per thread
__global__ __launch_bounds__(256) void scale_columns_f16_kernel(f16_t* W, const float* __restrict__ gain, size_t n8, int K,
                                                               uint32_t* overflow) {
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n8) return;
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    h8* p = reinterpret_cast<h8*>(W) + i;
    h8 w = *p;
    const int k0 = static_cast<int>((i * 8) % static_cast<size_t>(K));   // K is a multiple of 8
    bool over = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = static_cast<float>(w[e]) * gain[k0 + e];
        over |= fabsf(v) > 65504.0f;
        w[e] = static_cast<f16_t>(v);
    }
    *p = w;
    if (over) atomicOr(overflow, 1u);
}

void launch_scale_columns_f16(void* W, const float* gain, int32_t N, int32_t K, uint32_t* overflow, hipStream_t st) {
    const size_t n8 = static_cast<size_t>(N) * K / 8;
    launch(scale_columns_f16_kernel, dim3(static_cast<unsigned>((n8 + 255) / 256)), dim3(256), 0, st,
           static_cast<f16_t*>(W), gain, n8, K, overflow);
}

__global__ __launch_bounds__(256) void to_half_kernel(const float* __restrict__ x, f16_t* __restrict__ out, size_t n4,
                                                      uint32_t* oflow) {
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n4) return;
    const float4 t = reinterpret_cast<const float4*>(x)[i];
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    h4 o;
    o[0] = store_cast<f16_t>(t.x, oflow); o[1] = store_cast<f16_t>(t.y, oflow);
    o[2] = store_cast<f16_t>(t.z, oflow); o[3] = store_cast<f16_t>(t.w, oflow);
    reinterpret_cast<h4*>(out)[i] = o;
}

void launch_to_half(const float* x, void* out, size_t n, uint32_t* oflow, hipStream_t st) {
    const size_t n4 = n / 4;
    launch(to_half_kernel, dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0, st, x, static_cast<f16_t*>(out), n4, oflow);
}

// One-time kernel attribute calls happen inside the launchers; their first failure is kept here.
static std::atomic<int> g_attr_error{static_cast<int>(hipSuccess)};
static std::atomic<bool> g_attr_injected{false};
hipError_t kernel_attribute_error() {
    if (g_attr_injected.load()) return hipErrorInvalidValue;
    return static_cast<hipError_t>(g_attr_error.load());
}
void inject_kernel_attribute_error(bool on) { g_attr_injected.store(on); }
void note_kernel_attribute(hipError_t e) {
    int none = static_cast<int>(hipSuccess);
    if (e != hipSuccess) g_attr_error.compare_exchange_strong(none, static_cast<int>(e));
}

// bf16 -> half, in place, 8 elements per thread
__global__ __launch_bounds__(256) void bf16_to_f16_kernel(uint16_t* buf, size_t n8, uint32_t* overflow) {
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n8) return;
    uint4* p = reinterpret_cast<uint4*>(buf) + i;
    const uint4 w = *p;
    const uint32_t in[4] = {w.x, w.y, w.z, w.w};
    uint32_t out[4];
    bool over = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float lo = __uint_as_float(in[j] << 16), hi = __uint_as_float(in[j] & 0xFFFF0000u);
        over = over || fabsf(lo) > 65504.f || fabsf(hi) > 65504.f;
        const f16_t hl = static_cast<f16_t>(lo), hh = static_cast<f16_t>(hi);
        out[j] = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hl)) |
                 (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hh)) << 16);
    }
    *p = make_uint4(out[0], out[1], out[2], out[3]);
    if (over) *overflow = 1u;
}

void launch_bf16_to_f16(void* buf, size_t n, uint32_t* overflow, hipStream_t st) {
    const size_t n8 = n / 8;  // matrices here have a multiple of 8 elements per row
    launch(bf16_to_f16_kernel, dim3(static_cast<unsigned>((n8 + 255) / 256)), dim3(256), 0, st,
                       static_cast<uint16_t*>(buf), n8, overflow);
}

__global__ void table_update_kernel(int32_t* table, TableUpdate u) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < u.n) table[u.idx[i]] = u.val[i];
}

void launch_table_update(int32_t* table, const TableUpdate& u, hipStream_t st) {
    launch(table_update_kernel, dim3(1), dim3(128), 0, st, table, u);
}

// ---------------------------------------------------------------------------------------
// The ends of a model around its decoder layers: token embedding lookup and greedy choice.
// ---------------------------------------------------------------------------------------
template <typename WT>
__global__ __launch_bounds__(256) void embed_kernel(const WT* __restrict__ table, int V, int d, TokenIds by_value,
                                                    const int32_t* __restrict__ ids_dev, float* __restrict__ x_out,
                                                    uint32_t* bad) {
    constexpr int VEC = Elem<WT>::VEC;
    const int i = blockIdx.x;
    int id = ids_dev ? ids_dev[i] : by_value.id[i];
    if (id < 0 || id >= V) {
        if (threadIdx.x == 0) atomicOr(bad, 1u);
        id = id < 0 ? 0 : V - 1;
    }
    const WT* row = table + static_cast<size_t>(id) * d;
    float* out = x_out + static_cast<size_t>(i) * d;
    for (int c = threadIdx.x; c < d / VEC; c += 256) {
        Vec16<WT> w;
        w.load(row + static_cast<size_t>(c) * VEC);
#pragma unroll
        for (int e = 0; e < VEC; e += 4) {
            float4 o;
            o.x = w.v[e]; o.y = w.v[e + 1]; o.z = w.v[e + 2]; o.w = w.v[e + 3];
            *reinterpret_cast<float4*>(out + static_cast<size_t>(c) * VEC + e) = o;
        }
    }
}

void launch_embed(const void* table, int32_t dt, int32_t V, int32_t d, const TokenIds* by_value, const int32_t* ids_dev,
                  int32_t n, float* x_out, uint32_t* bad, hipStream_t st) {
    TokenIds none{};
    const TokenIds& ids = by_value ? *by_value : none;
    if (dt == DT_F32)
        launch(embed_kernel<float>, dim3(n), dim3(256), 0, st, static_cast<const float*>(table), V, d, ids, ids_dev, x_out, bad);
    else
        launch(embed_kernel<f16_t>, dim3(n), dim3(256), 0, st, static_cast<const f16_t*>(table), V, d, ids, ids_dev, x_out, bad);
}

__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int V, int32_t* __restrict__ out) {
    const float* row = logits + static_cast<size_t>(blockIdx.x) * V;
    float best = -INFINITY;
    int at = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 256) {
        const float v = row[i];
        if (v > best || (v == best && i < at)) { best = v; at = i; }   // NaN compares false: skipped
    }
    // lowest index among equal maxima, in every reduction step
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ob = __shfl_xor(best, off, 64);
        const int oa = __shfl_xor(at, off, 64);
        if (ob > best || (ob == best && oa < at)) { best = ob; at = oa; }
    }
    __shared__ float s_b[4];
    __shared__ int s_a[4];
    if ((threadIdx.x & 63) == 0) { s_b[threadIdx.x >> 6] = best; s_a[threadIdx.x >> 6] = at; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w)
            if (s_b[w] > best || (s_b[w] == best && s_a[w] < at)) { best = s_b[w]; at = s_a[w]; }
        out[blockIdx.x] = at == 0x7fffffff ? 0 : at;
    }
}

void launch_argmax(const float* logits, int32_t n, int32_t V, int32_t* out, hipStream_t st) {
    launch(argmax_kernel, dim3(n), dim3(256), 0, st, logits, V, out);
}

}  // namespace shk
