// Prefill-phase kernels (EdgeShard Sec. 2: the whole prompt is consumed at once and fills
// the KV cache).  The projections are dense contractions and run on the matrix cores
// (MFMA) from LDS-staged tiles; attention runs QK^T and PV on the matrix cores with the
// softmax statistics kept per lane and merged with one wavefront shuffle.
#include "kernels.hpp"

#include <mutex>

namespace shk {

// ---------------------------------------------------------------------------------------
// RMSNorm of rows: out = x * rsqrt(mean(x^2) + eps) * gain.  One workgroup per row.  Rows of
// up to 8192 elements (every Llama2 width) are held in registers: all loads of the row and of
// the gains go out at once and the row is read once; wider rows take two passes.
// ---------------------------------------------------------------------------------------
template <typename OT>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      float eps, OT* __restrict__ out, int d) {
    constexpr int NV = 8;   // float4 per thread in the register path
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* xr = x + static_cast<size_t>(blockIdx.x) * d;
    OT* orow = out + static_cast<size_t>(blockIdx.x) * d;
    const bool in_regs = d <= 1024 * NV;
    float4 v[NV], g[NV];
    float ssq = 0.f;
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = tid * 4 + i * 1024;
            v[i] = c < d ? *reinterpret_cast<const float4*>(xr + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = tid * 4 + i * 1024;
            g[i] = c < d ? *reinterpret_cast<const float4*>(gain + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) ssq += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    } else {
        for (int c = tid * 4; c < d; c += 1024) {
            const float4 t = *reinterpret_cast<const float4*>(xr + c);
            ssq += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
        }
    }
    __shared__ float s_part[4];
    ssq = wave_sum(ssq);
    if (lane == 0) s_part[wave] = ssq;
    __syncthreads();
    const float tot = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
    const float r = 1.0f / sqrtf(tot / static_cast<float>(d) + eps);
    auto put = [&](int c, const float4& t, const float4& gg) {
        orow[c] = Elem<OT>::from_f32(t.x * r * gg.x);
        orow[c + 1] = Elem<OT>::from_f32(t.y * r * gg.y);
        orow[c + 2] = Elem<OT>::from_f32(t.z * r * gg.z);
        orow[c + 3] = Elem<OT>::from_f32(t.w * r * gg.w);
    };
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = tid * 4 + i * 1024;
            if (c < d) put(c, v[i], g[i]);
        }
    } else {
        for (int c = tid * 4; c < d; c += 1024)
            put(c, *reinterpret_cast<const float4*>(xr + c), *reinterpret_cast<const float4*>(gain + c));
    }
}

void launch_rmsnorm(const float* x, const float* gain, float eps, void* out, int32_t out_dtype,
                    int32_t M, int32_t d, hipStream_t st) {
    if (out_dtype == DT_F32)
        launch(rmsnorm_kernel<float>, dim3(M), dim3(256), 0, st, x, gain, eps, static_cast<float*>(out), d);
    else
        launch(rmsnorm_kernel<f16_t>, dim3(M), dim3(256), 0, st, x, gain, eps, static_cast<f16_t*>(out), d);
}

// ---------------------------------------------------------------------------------------
// Shared epilogue of the prefill GEMMs.  The GEMMs compute the TRANSPOSED product
// D[n][m] = sum_k W[n][k] A[m][k], so that in the 32x32 MFMA result layout a lane holds
// one activation row m and four consecutive output features n..n+3: the element pairs
// RoPE and SwiGLU work on sit in one lane, and results leave as 16-byte stores.
// `val` = the four features n4..n4+3 (n4 % 4 == 0) of row m.
// ---------------------------------------------------------------------------------------
template <typename ET>
__device__ __forceinline__ void gemm_epilogue(const PrefillGemm& a, int m, int n4, const float val[4]) {
    if (m >= a.M || n4 >= a.N) return;
    if (a.epi == EPI_PARTIAL) {
        float4 o; o.x = val[0]; o.y = val[1]; o.z = val[2]; o.w = val[3];
        *reinterpret_cast<float4*>(a.out + static_cast<size_t>(m) * a.N + n4) = o;
        return;
    }
    // EPI_SWIGLU (the residual and the QKV epilogues are written out per tile below)
    const int F = a.N / 2;
    ET* op = static_cast<ET*>(a.out_act) + static_cast<size_t>(m) * F + n4 / 2;
    op[0] = store_cast<ET>(val[0] / (1.0f + expf(-val[0])) * val[1], a.oflow);
    op[1] = store_cast<ET>(val[2] / (1.0f + expf(-val[2])) * val[3], a.oflow);
}

// Epilogue of a wave's TN x TM accumulator tiles (tile (i, j): features n_base + 32 i .., rows
// m_base + 32 j + l32; register v of a lane is feature 8 (v / 4) + 4 half + v % 4 of its tile).
// The residual epilogue reads before it writes, and output and residual may be the same buffer,
// so the compiler keeps every read behind the write before it: one memory round trip per 16
// bytes, 32 of them in a row at the end of a 256 x 256 tile while the matrix cores idle (the
// 70B-shape O projection ran 19 % below the gate/up projection for that reason alone).  Here
// the four reads of a 32 x 32 tile go out together, and the next tile's reads before the
// current tile's writes.
template <typename ET, int TN, int TM>
__device__ __forceinline__ void gemm_tile_epilogues(const PrefillGemm& a, const SeqBatch& sb, const f32x16 (&acc)[TN][TM],
                                                    int n_base, int m_base, int l32, int half) {
    if (a.epi == EPI_RESID) {
        float4 r[2][4];
        auto addr = [&](int t, int vq, bool* ok) {
            const int i = t / TM, j = t % TM;
            const int n4 = n_base + i * 32 + vq * 8 + half * 4, m = m_base + j * 32 + l32;
            *ok = m < a.M && n4 < a.N;
            return static_cast<size_t>(m) * a.N + n4;
        };
        auto fetch = [&](int t) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                bool ok;
                const size_t at = addr(t, vq, &ok);
                r[t & 1][vq] = ok ? *reinterpret_cast<const float4*>(a.resid + at) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        };
        fetch(0);
#pragma unroll
        for (int t = 0; t < TN * TM; ++t) {
            if (t + 1 < TN * TM) fetch(t + 1);
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                bool ok;
                const size_t at = addr(t, vq, &ok);
                if (!ok) continue;
                const f32x16& c = acc[t / TM][t % TM];
                const float4 x = r[t & 1][vq];
                float4 o;
                o.x = x.x + c[vq * 4]; o.y = x.y + c[vq * 4 + 1]; o.z = x.z + c[vq * 4 + 2]; o.w = x.w + c[vq * 4 + 3];
                *reinterpret_cast<float4*>(a.out + at) = o;
            }
        }
        return;
    }
    if (a.epi == EPI_QKV) {
        // What depends on the ROW only - sequence, position, rotation-table row, cache row of the
        // token's page - is worked out once per row tile (the block-table read included, and only
        // if the wave's features reach into the K / V range), not once per 16 bytes of output; the
        // four rotation-table reads of a 32 x 32 tile go out together.
        const int dh = a.kv.dh, nq = a.hq * dh, nk = a.kv.hkv * dh;
        const bool wave_has_kv = n_base + TN * 32 > nq;
        const float2* rope_row[TM];
        size_t cache_row[TM];   // row of (token, kv head 0) in units of dh elements; head hk adds hk * page
        bool row_ok[TM];
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m_base + j * 32 + l32;
            row_ok[j] = m < a.M;
            const int mm = row_ok[j] ? m : a.M - 1;
            const int b = mm / a.T, pos = sb.pos[b] + (mm - b * a.T);
            rope_row[j] = a.rope + static_cast<size_t>(pos) * (dh / 2);
            cache_row[j] = wave_has_kv ? kv_row_div(a.kv, a.kv.block_table + static_cast<size_t>(sb.seq[b]) * a.kv.max_pages, pos, 0) : 0;
        }
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int m = m_base + j * 32 + l32;
                float4 cs[4];   // (cos, sin) of the two pairs of each 16-byte group
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int n4 = n_base + i * 32 + vq * 8 + half * 4;
                    cs[vq] = (n4 < nq + nk && n4 < a.N) ? *reinterpret_cast<const float4*>(rope_row[j] + (n4 % dh) / 2)
                                                       : make_float4(1.f, 0.f, 1.f, 0.f);
                }
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int n4 = n_base + i * 32 + vq * 8 + half * 4;
                    if (!row_ok[j] || n4 >= a.N) continue;
                    const f32x16& c = acc[i][j];
                    const float v0 = c[vq * 4], v1 = c[vq * 4 + 1], v2 = c[vq * 4 + 2], v3 = c[vq * 4 + 3];
                    const bool rot = n4 < nq + nk;   // v is not rotated
                    const float r0 = rot ? v0 * cs[vq].x - v1 * cs[vq].y : v0, r1 = rot ? v0 * cs[vq].y + v1 * cs[vq].x : v1;
                    const float r2 = rot ? v2 * cs[vq].z - v3 * cs[vq].w : v2, r3 = rot ? v2 * cs[vq].w + v3 * cs[vq].z : v3;
                    if (n4 < nq) {
                        *reinterpret_cast<float4*>(a.q + static_cast<size_t>(m) * nq + n4) = make_float4(r0, r1, r2, r3);
                        continue;
                    }
                    const bool is_k = n4 < nq + nk;
                    const int f = n4 - nq - (is_k ? 0 : nk), hk = f / dh, e = f - hk * dh;
                    ET* dst = static_cast<ET*>(is_k ? a.kv.k : a.kv.v) + (cache_row[j] + static_cast<size_t>(hk) * a.kv.page) * dh + e;
                    dst[0] = store_cast<ET>(r0, a.oflow); dst[1] = store_cast<ET>(r1, a.oflow);
                    dst[2] = store_cast<ET>(r2, a.oflow); dst[3] = store_cast<ET>(r3, a.oflow);
                }
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int n4 = n_base + i * 32 + vq * 8 + half * 4;
                const int m = m_base + j * 32 + l32;
                const float val[4] = {acc[i][j][vq * 4], acc[i][j][vq * 4 + 1], acc[i][j][vq * 4 + 2], acc[i][j][vq * 4 + 3]};
                gemm_epilogue<ET>(a, m, n4, val);
            }
}

// ---------------------------------------------------------------------------------------
// GEMM on the matrix cores, fp32 accumulation: v_mfma_f32_32x32x2_f32 for fp32 operands,
// v_mfma_f32_32x32x16_f16 for half operands.
// Workgroup tile BN (features) x BM (rows), four waves in a 2x2 arrangement, each owning
// (BN/2) x (BM/2) as 32x32 MFMA tiles.  K is walked in steps of ROWDW dwords per row (64 or
// 128 bytes) through two LDS stages: the global loads of step k+1 are in flight while step k
// is multiplied.  LDS rows are k-contiguous.  Within a 32-byte k group the lane with
// half = lane/32 supplies the 16 bytes at offset 16*half - for fp32 that is a permutation
// of k (the same on both operands, so the sum over k is unchanged), for half it is the
// instruction's native operand layout.
//
// LDS layout: PITCH is the row pitch in dwords.  PITCH == ROWDW selects the unpadded,
// XOR-swizzled layout: 16-byte chunk c of row r is stored at chunk c ^ g(r), g(r) = (r/4)%4
// for 4-chunk rows and (r/2)%8 for 8-chunk rows.  Measured on MI355X (SQ_LDS_BANK_CONFLICT):
// LDS serves 16-byte reads from 16 lanes per clock over 64 banks and 16-byte writes from 8
// lanes per clock over 32 banks; the swizzle is conflict-free for both, while a padded pitch
// (ROWDW + 4) is conflict-free for the reads only (its stores, two rows per 8 lanes, collide:
// a third of the LDS cycles at ROWDW = 16).
// ---------------------------------------------------------------------------------------

// Tile order.  Workgroups are dealt round-robin to the 8 XCDs (blockIdx % 8), each with its
// own L2; every XCD gets a contiguous run of the tile sequence, and the sequence walks the
// row tiles of a band of at most 8 before it moves to the next feature tile.  The workgroups
// resident on an XCD at one time then form a block of about 8 x 4 tiles that shares its W
// and its activation rows through that L2 (one feature tile at a time would re-stream all
// activation rows from beyond the L2 for every feature tile once M is large).
__device__ __forceinline__ bool tile_origin(int tiles_m, int tiles_total, int bn, int bm, int* n0, int* m0) {
    const int per_xcd = (tiles_total + 7) / 8;
    const int t = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (t >= tiles_total) return false;
    const int tiles_n = tiles_total / tiles_m;
    const int band = t / (8 * tiles_n), first_m = band * 8;
    const int gm = min(tiles_m - first_m, 8);
    const int r = t - band * 8 * tiles_n;
    *m0 = (first_m + r % gm) * bm;
    *n0 = (r / gm) * bn;
    return true;
}

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

template <typename T>
__device__ __forceinline__ void mfma_chunk(const float4& w, const float4& x, f32x16& acc);
template <>
__device__ __forceinline__ void mfma_chunk<float>(const float4& w, const float4& x, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.x, x.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.y, x.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.z, x.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(w.w, x.w, acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mfma_chunk<f16_t>(const float4& w, const float4& x, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, w), __builtin_bit_cast(f16x8_t, x),
                                                 acc, 0, 0, 0);
}

template <typename T, int BN, int BM, int ROWDW, int PITCH>
__global__ __launch_bounds__(256) void gemm_kernel(PrefillGemm a, SeqBatch sb, int tiles_m, int tiles_total) {
    constexpr int VEC = Elem<T>::VEC;          // elements per 16 bytes
    constexpr int CH = ROWDW / 4;              // 16-byte chunks per row per step
    constexpr int BK = CH * VEC;               // elements of k per step
    constexpr int TN = BN / 64, TM = BM / 64;  // MFMA tiles per wave
    constexpr int LW = BN * CH / 256, LX = BM * CH / 256;  // 16-byte loads per thread per stage
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* const sW0 = smem;                               // [2][BN * PITCH]
    float* const sX0 = smem + 2 * BN * PITCH;              // [2][BM * PITCH]

    int n0, m0;
    if (!tile_origin(tiles_m, tiles_total, BN, BM, &n0, &m0)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave >> 1, wm = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;
    // dword offset of 16-byte chunk c of tile row r
    auto lds_at = [](int r, int c) {
        if constexpr (PITCH == ROWDW) return r * PITCH + ((c ^ (CH == 4 ? (r >> 2) & 3 : (r >> 1) & 7)) << 2);
        else return r * PITCH + (c << 2);
    };
    typedef typename ActOf<T>::type AT;  // activation type (same size as T)
    const T* __restrict__ W = static_cast<const T*>(a.W);
    const AT* __restrict__ X = static_cast<const AT*>(a.A);

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    float4 gw[LW], gx[LX];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int idx = tid + 256 * i, row = idx / CH, k = k0 + (idx % CH) * VEC;
            const bool ok = (n0 + row < a.N) && (k < a.K);
            gw[i] = ok ? *reinterpret_cast<const float4*>(W + static_cast<size_t>(n0 + row) * a.K + k)
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            const int idx = tid + 256 * i, row = idx / CH, k = k0 + (idx % CH) * VEC;
            const bool ok = (m0 + row < a.M) && (k < a.K);
            gx[i] = ok ? *reinterpret_cast<const float4*>(X + static_cast<size_t>(m0 + row) * a.K + k)
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto sstore = [&](int stage) {
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<float4*>(&sW0[stage * BN * PITCH + lds_at(idx / CH, idx % CH)]) = gw[i];
        }
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            const int idx = tid + 256 * i;
            *reinterpret_cast<float4*>(&sX0[stage * BM * PITCH + lds_at(idx / CH, idx % CH)]) = gx[i];
        }
    };

    const int ksteps = (a.K + BK - 1) / BK;
    gload(0);
    sstore(0);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const int stage = ks & 1;
        if (ks + 1 < ksteps) gload((ks + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < ROWDW / 8; ++kk) {
            float4 fw[TN], fx[TM];
#pragma unroll
            for (int i = 0; i < TN; ++i)
                fw[i] = *reinterpret_cast<const float4*>(
                    &sW0[stage * BN * PITCH + lds_at(wn * (BN / 2) + i * 32 + l32, kk * 2 + half)]);
#pragma unroll
            for (int j = 0; j < TM; ++j)
                fx[j] = *reinterpret_cast<const float4*>(
                    &sX0[stage * BM * PITCH + lds_at(wm * (BM / 2) + j * 32 + l32, kk * 2 + half)]);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) mfma_chunk<T>(fw[i], fx[j], acc[i][j]);
        }
        if (ks + 1 < ksteps) sstore(stage ^ 1);
        __syncthreads();
    }

    gemm_tile_epilogues<AT, TN, TM>(a, sb, acc, n0 + wn * (BN / 2), m0 + wm * (BM / 2), l32, half);
}

template <typename T, int BN, int BM, int ROWDW, int PITCH>
static void launch_gemm(const PrefillGemm& a, const SeqBatch& sb, hipStream_t st) {
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int grid = ((total + 7) / 8) * 8;
    constexpr size_t lds = 2u * (BN + BM) * PITCH * sizeof(float);
    static std::once_flag once;  // more than 64 KB of LDS per workgroup is an opt-in
    std::call_once(once, [] {
        note_kernel_attribute(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<T, BN, BM, ROWDW, PITCH>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    });
    launch((gemm_kernel<T, BN, BM, ROWDW, PITCH>), dim3(grid), dim3(256), lds, st, a, sb, tiles_m, total);
}

// ---------------------------------------------------------------------------------------
// GEMM with direct global->LDS loads (global_load_lds_dwordx4, gfx950) and a
// ring of STAGES k-steps in LDS.  The register-staged kernel above keeps one k-step in
// flight per workgroup; at the matrix cores' half-precision rate that is a fraction of the
// bytes the memory latency asks for, and the counters show its waves waiting on their own
// loads.  Here the loads of k-step ks + STAGES - 1 are issued while step ks is multiplied,
// they occupy no registers, and one barrier per step both publishes a landed stage and
// frees the one just consumed.
// A wave-level load writes 64 lanes x 16 bytes to consecutive LDS addresses, i.e. 64/CH whole
// rows of a stage; the XOR swizzle is applied on the global side (lane l fetches the chunk
// that belongs in its LDS slot).  Rows past the matrix edge are clamped to the last row:
// they feed accumulators that are never stored.  K must be a multiple of the k-step.
// The loads are inline assembly because the compiler, for its own direct-to-LDS builtin,
// waits for every outstanding load before any LDS read; waits here are explicit.
// ---------------------------------------------------------------------------------------

template <typename T, int BN, int BM, int ROWDW, int STAGES, int WN, int WM>
__global__ __launch_bounds__(64 * WN * WM) void gemm_dma_kernel(PrefillGemm a, SeqBatch sb, int tiles_m, int tiles_total) {
    constexpr int NW = WN * WM;                  // waves per workgroup
    constexpr int CH = ROWDW / 4;                // 16-byte chunks per row per step
    constexpr int VEC = Elem<T>::VEC;            // elements per 16 bytes
    constexpr int BK = CH * VEC;                 // elements of k per step
    constexpr int TN = BN / WN / 32, TM = BM / WM / 32;  // MFMA tiles per wave
    constexpr int RPC = 64 / CH;                 // rows per wave-level load (1 KB)
    constexpr int NCW = BN / RPC, NCX = BM / RPC, NPER = (NCW + NCX) / NW;
    constexpr int STAGE_DW = (BN + BM) * ROWDW;
    static_assert((NCW + NCX) % NW == 0, "loads must divide evenly over the waves");
    static_assert(NPER * (STAGES - 1) < 64, "vmcnt is a 6-bit counter");
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)smem));

    int n0, m0;
    if (!tile_origin(tiles_m, tiles_total, BN, BM, &n0, &m0)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave / WM, wm = wave % WM;
    const int l32 = lane & 31, half = lane >> 5;
    auto swz = [](int r) { return CH == 4 ? (r >> 2) & 3 : (r >> 1) & 7; };
    auto lds_at = [&](int r, int c) { return r * ROWDW + ((c ^ swz(r)) << 2); };

    typedef typename ActOf<T>::type AT;          // activation type (same size as T)
    const T* __restrict__ W = static_cast<const T*>(a.W);
    const T* __restrict__ X = static_cast<const T*>(a.A);
    const T* src[NPER];
    uint32_t dst[NPER];
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
        const int c = wave + NW * i;             // this wave's i-th load of a stage
        const bool is_w = c < NCW;
        const int cc = is_w ? c : c - NCW;
        const int row = cc * RPC + lane / CH;
        const int chunk = (lane % CH) ^ swz(row);
        const int grow = is_w ? min(n0 + row, a.N - 1) : min(m0 + row, a.M - 1);
        src[i] = (is_w ? W : X) + static_cast<size_t>(grow) * a.K + chunk * VEC;
        dst[i] = lds0 + (is_w ? 0 : BN * ROWDW * 4) + cc * 1024;
    }
    // split K: workgroup row blockIdx.y of the grid takes k-steps [ks_lo, ks_hi) and stores its
    // partial sums to slice blockIdx.y of a.part; splitk_reduce_kernel adds the slices in order
    PrefillGemm ae = a;
    int ks_lo = 0, ks_hi = a.K / BK;
    if (a.kslices > 1) {
        const int all = a.K / BK, slice = blockIdx.y;
        ks_lo = static_cast<int>(static_cast<long>(all) * slice / a.kslices);
        ks_hi = static_cast<int>(static_cast<long>(all) * (slice + 1) / a.kslices);
        ae.epi = EPI_PARTIAL;
        ae.out = a.part + static_cast<size_t>(slice) * a.M * a.N;
#pragma unroll
        for (int i = 0; i < NPER; ++i) src[i] += static_cast<size_t>(ks_lo) * BK;
    }
    const int ksteps = ks_hi - ks_lo;
    auto issue = [&](int ks) {                   // k-step ks -> stage ks % STAGES
        const int kc = ks < ksteps ? ks : ksteps - 1;   // past the end: a harmless reload into a free stage
        const uint32_t sb0 = static_cast<uint32_t>(ks % STAGES) * (STAGE_DW * 4);
#pragma unroll
        for (int i = 0; i < NPER; ++i) lds_dma16(src[i] + static_cast<size_t>(kc) * BK, dst[i] + sb0);
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s);
    for (int ks = 0; ks < ksteps; ++ks) {
        wait_vmcnt<NPER*(STAGES - 2)>();         // this wave's loads of step ks have landed
        __syncthreads();                         // ... everyone's; and stage (ks-1) % STAGES is free
        const float* sW = smem + (ks % STAGES) * STAGE_DW;
        const float* sX = sW + BN * ROWDW;
        // fragments of k-group kk+1 are fetched while the matrix cores work on group kk
        float4 fw[2][TN], fx[2][TM];
        auto fetch = [&](int kk, int buf) {
#pragma unroll
            for (int i = 0; i < TN; ++i)
                fw[buf][i] = *reinterpret_cast<const float4*>(&sW[lds_at(wn * (BN / WN) + i * 32 + l32, kk * 2 + half)]);
#pragma unroll
            for (int j = 0; j < TM; ++j)
                fx[buf][j] = *reinterpret_cast<const float4*>(&sX[lds_at(wm * (BM / WM) + j * 32 + l32, kk * 2 + half)]);
        };
        fetch(0, 0);
        issue(ks + STAGES - 1);                  // issued under the latency of the first fetch
#pragma unroll
        for (int kk = 0; kk < ROWDW / 8; ++kk) {
            if (kk + 1 < ROWDW / 8) fetch(kk + 1, (kk + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);   // keep the fetch ahead of the multiplies
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) mfma_chunk<T>(fw[kk & 1][i], fx[kk & 1][j], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_vmcnt<0>();                             // the reloads past the end

    gemm_tile_epilogues<AT, TN, TM>(ae, sb, acc, n0 + wn * (BN / WN), m0 + wm * (BM / WM), l32, half);
}

template <typename T, int BN, int BM, int ROWDW, int STAGES, int WN, int WM>
static void launch_gemm_dma(const PrefillGemm& a, const SeqBatch& sb, hipStream_t st) {
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int grid = ((total + 7) / 8) * 8;
    constexpr size_t lds = static_cast<size_t>(STAGES) * (BN + BM) * ROWDW * sizeof(float);
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    static std::once_flag once;  // more than 64 KB of LDS per workgroup is an opt-in
    std::call_once(once, [] {
        note_kernel_attribute(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_dma_kernel<T, BN, BM, ROWDW, STAGES, WN, WM>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    });
    launch(gemm_dma_kernel<T, BN, BM, ROWDW, STAGES, WN, WM>, dim3(grid, a.kslices > 1 ? a.kslices : 1), dim3(64 * WN * WM), lds,
           st, a, sb, tiles_m, total);
}

// out = resid + (slice 0 + slice 1 + ...), four elements per thread
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int slices, size_t slice_elems,
                                                            const float* resid, float* out) {
    const size_t i = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
    if (i >= slice_elems) return;
    float4 acc = *reinterpret_cast<const float4*>(part + i);
    for (int s = 1; s < slices; ++s) {
        const float4 t = *reinterpret_cast<const float4*>(part + static_cast<size_t>(s) * slice_elems + i);
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    const float4 r = *reinterpret_cast<const float4*>(resid + i);
    acc.x += r.x; acc.y += r.y; acc.z += r.z; acc.w += r.w;
    *reinterpret_cast<float4*>(out + i) = acc;
}

// Tile choice.  A compute unit holds `occ` workgroups of a variant at once and gets
// ceil(tiles / 256) of them; what a variant achieves depends strongly on how many of its
// workgroups are resident together (one alone cannot hide the latency of its own loads), so
// the tail of a launch - the last n % occ tiles of a compute unit - runs at a lower rate.
// rate[r-1] is the measured throughput (TFLOP/s, whole chip, Llama2 shapes at M = 512..4096)
// with r workgroups resident per compute unit; the estimate below adds up full groups and the
// tail and the cheapest variant is launched.
struct GemmVariant {
    int bn, bm, occ;
    float rate[3];
};

static int pick_variant(const GemmVariant* v, int count, int M, int N) {
    int best = 0;
    double best_t = 0;
    for (int c = 0; c < count; ++c) {
        const long tiles = static_cast<long>((M + v[c].bm - 1) / v[c].bm) * ((N + v[c].bn - 1) / v[c].bn);
        const long n = (tiles + 255) / 256;
        const double w = static_cast<double>(v[c].bn) * v[c].bm;
        const long tail = n % v[c].occ;
        double t = static_cast<double>(n - tail) * w / v[c].rate[v[c].occ - 1];
        if (tail) t += static_cast<double>(tail) * w / v[c].rate[tail - 1];
        if (c == 0 || t < best_t) { best = c; best_t = t; }
    }
    return best;
}

// Every variant the launchers below can take, by name: the selection (choose_prefill_gemm) is
// a pure host function of the shape, so that tests can ask which variant a shape lands on.
enum GemmId {
    G32_DMA_128x128, G32_DMA_128x64, G32_DMA_192x64, G32_DMA_192x128, G32_DMA_128x64_K32, G32_DMA_128x64_SPLITK, G32_DMA_128x128_SPLITK,
    G32_REG_128x128, G32_REG_128x64,
    G16_DMA_256x256, G16_DMA_256x128, G16_DMA_128x128, G16_DMA_128x64, G16_DMA_384x128, G16_DMA_192x256, G16_DMA_64x64,
    G16_DMA_128x64_SPLITK, G16_DMA_128x128_SPLITK, G16_REG_128x128_K32, G16_REG_128x128_K64, G16_REG_128x64,
    GEMM_ID_COUNT
};
static const char* const GEMM_NAMES[GEMM_ID_COUNT] = {
    "f32 dma 128x128", "f32 dma 128x64", "f32 dma 192x64", "f32 dma 192x128", "f32 dma 128x64 k32", "f32 dma 128x64 split-k", "f32 dma 128x128 split-k",
    "f32 reg 128x128", "f32 reg 128x64",
    "f16 dma 256x256", "f16 dma 256x128", "f16 dma 128x128", "f16 dma 128x64", "f16 dma 384x128", "f16 dma 192x256", "f16 dma 64x64",
    "f16 dma 128x64 split-k", "f16 dma 128x128 split-k", "f16 reg 128x128 k32", "f16 reg 128x128 k64", "f16 reg 128x64",
};
const char* prefill_gemm_variant_name(int id) { return id >= 0 && id < GEMM_ID_COUNT ? GEMM_NAMES[id] : nullptr; }

// Split K for a projection back to d_model with too few output tiles for the chip (13B shape,
// M = 256: 80 tiles of 128 x 128): K goes over S <= 4 rows of workgroups (grid y) so that tiles x S
// comes out at one workgroup per compute unit or just below, each slice at least 512 elements of
// K, into an fp32 scratch, and splitk_reduce_kernel adds slices and residual in slice order.  Of
// the 128 x 128 and the 128 x 64 tile the one that puts more workgroups on the chip that way is
// taken, the larger on a tie.  Measured alone, half precision: 13B at M = 256, S = 3: O 36 -> 31 us,
// down 76 -> 60 us against 128 x 64 tiles with the same S; 7B down at M = 256 / 384 / 512:
// 51 -> 43, 84 -> 64, 84 -> 71 us; 13B at M = 128: 128 x 64 with S = 3, 23 us against 30 us with
// S = 4.  fp32, 7B: M = 128 O 138 -> 45 us, down 363 -> 109 us (128 x 64, S = 4); M = 256 O 136 -> 78,
// down 365 -> 189 us (128 x 128, S = 4); M = 512 (128 tiles of 128 x 128, S = 2) O 141, down 350 us
// against 146 and 355 us with two slices over 128 x 64 tiles and 141 and 367 us unsplit.  From 256
// tiles on a split loses.
// Returns 0 (no split), 64 or 128 (the tile's row count) and the slice count.
static int choose_split(int M, int N, int K, size_t part_cap, int* slices) {
    const size_t elems = static_cast<size_t>(M) * N;
    if (elems % 4 != 0) return 0;
    const long t64 = static_cast<long>((M + 63) / 64) * ((N + 127) / 128);
    const long t128 = static_cast<long>((M + 127) / 128) * ((N + 127) / 128);
    auto fit = [&](long tiles) {
        long S = 256 / tiles;
        if (S > 4) S = 4;
        if (S > K / 512) S = K / 512;
        while (S >= 2 && elems * static_cast<size_t>(S) > part_cap) --S;
        return S;
    };
    const long s128 = M > 64 ? fit(t128) : 0, s64 = fit(t64);
    if (s128 >= 2 && t128 * s128 >= t64 * s64) {
        *slices = static_cast<int>(s128);
        return 128;
    }
    if (s64 >= 2) {
        *slices = static_cast<int>(s64);
        return 64;
    }
    return 0;
}

int choose_prefill_gemm(int dt, int M, int N, int K, int epi, bool has_part, size_t part_cap, int* kslices) {
    *kslices = 1;
    const size_t elems = static_cast<size_t>(M) * N;
    const long t64 = static_cast<long>((M + 63) / 64) * ((N + 127) / 128);
    if (dt == DT_F32) {
        if (K % 16 == 0) {  // direct-to-LDS variants (k-step of 16 or 32)
            static const GemmVariant v[] = {{128, 128, 2, {100.f, 142.f, 0.f}},
                                            {128, 64, 3, {125.f, 120.f, 116.f}},
                                            {192, 64, 2, {118.f, 138.f, 0.f}},   // 12288 x 512: two tiles per unit, both resident
                                            {192, 128, 2, {136.f, 144.f, 0.f}},  // 22016 x 512: 460 tiles, at most two per unit
                                            {128, 64, 2, {116.f, 131.f, 0.f}}};  // k-step 32
            if (epi == EPI_RESID && has_part) {   // too few output tiles for the chip: see choose_split
                const int rows = choose_split(M, N, K, part_cap, kslices);
                if (rows) return rows == 128 ? G32_DMA_128x128_SPLITK : G32_DMA_128x64_SPLITK;
            }
            static const int ids[] = {G32_DMA_128x128, G32_DMA_128x64, G32_DMA_192x64, G32_DMA_192x128, G32_DMA_128x64_K32};
            return ids[pick_variant(v, K % 32 == 0 ? 5 : 4, M, N)];
        }
        static const GemmVariant v[] = {{128, 128, 3, {108.f, 128.f, 133.f}}, {128, 64, 3, {101.f, 119.f, 125.f}}};
        return pick_variant(v, 2, M, N) == 0 ? G32_REG_128x128 : G32_REG_128x64;
    }
    if (K % 64 == 0) {  // direct-to-LDS variants (k-step of 64)
        static const GemmVariant v[] = {{256, 256, 1, {1500.f, 0.f, 0.f}},
                                        {256, 128, 1, {1250.f, 0.f, 0.f}},
                                        {128, 128, 1, {1000.f, 0.f, 0.f}},
                                        {128, 64, 2, {650.f, 900.f, 0.f}},
                                        {384, 128, 1, {1300.f, 0.f, 0.f}},
                                        // 256 tiles for 12288 x 1024 and 460 for 22016 x 1024 (7B shapes at 1024 rows: 120 and
                                        // 203 us against 126 and 223 us with 384 x 128), 216 for 5120 x 2048
                                        {192, 256, 1, {1380.f, 0.f, 0.f}},
                                        {64, 64, 1, {330.f, 0.f, 0.f}}};     // a few dozen rows: more workgroups stream the weights
        if (epi == EPI_RESID && has_part) {   // too few output tiles for the chip: see choose_split
            const int rows = choose_split(M, N, K, part_cap, kslices);
            if (rows) return rows == 128 ? G16_DMA_128x128_SPLITK : G16_DMA_128x64_SPLITK;
        }
        static const int ids[] = {G16_DMA_256x256, G16_DMA_256x128, G16_DMA_128x128, G16_DMA_128x64, G16_DMA_384x128, G16_DMA_192x256, G16_DMA_64x64};
        return ids[pick_variant(v, 7, M, N)];
    }
    static const GemmVariant v[] = {{128, 128, 3, {390.f, 650.f, 850.f}},
                                    {128, 128, 2, {470.f, 800.f, 0.f}},
                                    {128, 64, 3, {270.f, 490.f, 700.f}}};
    static const int ids[] = {G16_REG_128x128_K32, G16_REG_128x128_K64, G16_REG_128x64};
    return ids[pick_variant(v, 3, M, N)];
}

void launch_prefill_gemm(const PrefillGemm& a, const SeqBatch& sb, hipStream_t st) {
    int kslices = 1;
    const int id = choose_prefill_gemm(a.dt, a.M, a.N, a.K, a.epi, a.part != nullptr, a.part_cap, &kslices);
    PrefillGemm as = a;
    as.kslices = kslices;
    switch (id) {
        case G32_DMA_128x128: launch_gemm_dma<float, 128, 128, 16, 4, 2, 2>(as, sb, st); break;
        case G32_DMA_128x64: launch_gemm_dma<float, 128, 64, 16, 4, 2, 2>(as, sb, st); break;
        case G32_DMA_192x64: launch_gemm_dma<float, 192, 64, 16, 4, 2, 2>(as, sb, st); break;
        case G32_DMA_192x128: launch_gemm_dma<float, 192, 128, 16, 4, 2, 2>(as, sb, st); break;
        case G32_DMA_128x64_K32: launch_gemm_dma<float, 128, 64, 32, 3, 2, 2>(as, sb, st); break;
        case G32_DMA_128x64_SPLITK: launch_gemm_dma<float, 128, 64, 16, 4, 2, 2>(as, sb, st); break;
        case G32_DMA_128x128_SPLITK: launch_gemm_dma<float, 128, 128, 16, 4, 2, 2>(as, sb, st); break;
        case G32_REG_128x128: launch_gemm<float, 128, 128, 16, 16>(as, sb, st); break;
        case G32_REG_128x64: launch_gemm<float, 128, 64, 32, 32>(as, sb, st); break;
        case G16_DMA_256x256: launch_gemm_dma<f16_t, 256, 256, 32, 2, 4, 2>(as, sb, st); break;
        case G16_DMA_256x128: launch_gemm_dma<f16_t, 256, 128, 32, 3, 4, 2>(as, sb, st); break;
        case G16_DMA_128x128: launch_gemm_dma<f16_t, 128, 128, 32, 3, 2, 2>(as, sb, st); break;
        case G16_DMA_128x64: launch_gemm_dma<f16_t, 128, 64, 32, 3, 2, 2>(as, sb, st); break;
        case G16_DMA_384x128: launch_gemm_dma<f16_t, 384, 128, 32, 2, 4, 2>(as, sb, st); break;
        case G16_DMA_192x256: launch_gemm_dma<f16_t, 192, 256, 32, 2, 2, 4>(as, sb, st); break;
        case G16_DMA_64x64: launch_gemm_dma<f16_t, 64, 64, 32, 6, 2, 2>(as, sb, st); break;
        case G16_DMA_128x64_SPLITK: launch_gemm_dma<f16_t, 128, 64, 32, 3, 2, 2>(as, sb, st); break;
        case G16_DMA_128x128_SPLITK: launch_gemm_dma<f16_t, 128, 128, 32, 3, 2, 2>(as, sb, st); break;
        case G16_REG_128x128_K32: launch_gemm<f16_t, 128, 128, 16, 16>(as, sb, st); break;
        case G16_REG_128x128_K64: launch_gemm<f16_t, 128, 128, 32, 32>(as, sb, st); break;
        default: launch_gemm<f16_t, 128, 64, 32, 32>(as, sb, st); break;
    }
    if (kslices > 1) {
        const size_t elems = static_cast<size_t>(a.M) * a.N;
        launch(splitk_reduce_kernel, dim3(static_cast<unsigned>((elems / 4 + 255) / 256)), dim3(256), 0, st,
               static_cast<const float*>(a.part), kslices, elems, a.resid, a.out);
    }
}

// ---------------------------------------------------------------------------------------
// Causal attention for the T new tokens of each sequence over its cache (positions
// 0 .. P+T-1).  One wave owns 32 query rows of one head; the four waves of a workgroup
// take four heads of the same query tile, so they carry equal work.  Per 32-key tile:
//   S^T[key][q] = sum_d K[key][d] Q[q][d]      (MFMA, K and Q fragments k-contiguous)
//   a lane then holds 16 keys of ONE query column: row max / row sum are in-lane
//   reductions plus a single shuffle with lane^32;
//   O^T[d][q] += sum_key V[key][d] P^T[key][q]  (MFMA; P^T is already in B-operand layout).
// ---------------------------------------------------------------------------------------
template <typename KT>
__device__ __forceinline__ float4 load4(const KT* p);
template <>
__device__ __forceinline__ float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <>
__device__ __forceinline__ float4 load4<f16_t>(const f16_t* p) {
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    const h4 t = *reinterpret_cast<const h4*>(p);
    return make_float4(static_cast<float>(t[0]), static_cast<float>(t[1]), static_cast<float>(t[2]), static_cast<float>(t[3]));
}

template <typename KT, typename OT, int DH>
__global__ __launch_bounds__(256) void prefill_attn_kernel(PrefillAttn a, SeqBatch sb) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int qt = gridDim.x - 1 - blockIdx.x;  // longest rows first
    const int h = blockIdx.y * 4 + wave;
    const int b = blockIdx.z;
    if (h >= a.hq) return;
    const int hk = h / (a.hq / a.kv.hkv);
    const int P = sb.pos[b];
    const int32_t* bt = a.kv.block_table + static_cast<size_t>(sb.seq[b]) * a.kv.max_pages;
    const KT* __restrict__ kp = static_cast<const KT*>(a.kv.k);
    const KT* __restrict__ vp = static_cast<const KT*>(a.kv.v);
    const int ctx = P + a.T;

    const int t_q = qt * 32 + l32;                // this lane's query row within the call
    const int t_ld = min(t_q, a.T - 1);
    const size_t qrow = (static_cast<size_t>(b) * a.T + t_ld) * a.hq * DH + h * DH;
    const float scale = 1.0f / sqrtf(static_cast<float>(DH));
    float4 qf[DH / 8];
#pragma unroll
    for (int j = 0; j < DH / 8; ++j) {
        qf[j] = *reinterpret_cast<const float4*>(a.q + qrow + j * 8 + half * 4);
        qf[j].x *= scale; qf[j].y *= scale; qf[j].z *= scale; qf[j].w *= scale;
    }
    f32x16 o[DH / 32];
#pragma unroll
    for (int j = 0; j < DH / 32; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[j][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const int pos_q = P + t_q;
    const int last_key = P + min(qt * 32 + 31, a.T - 1);

    for (int k0 = 0; k0 <= last_key; k0 += 32) {
        // S^T tile
        const int u = min(k0 + l32, ctx - 1);
        const size_t kat = kv_row_div(a.kv, bt, u, hk) * DH + half * 4;
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int j = 0; j < DH / 8; ++j) {
            const float4 kf = load4<KT>(kp + kat + j * 8);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.x, qf[j].x, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.y, qf[j].y, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.z, qf[j].z, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.w, qf[j].w, s, 0, 0, 0);
        }
        // causal mask + running softmax for this lane's query column
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = k0 + (v >> 2) * 8 + half * 4 + (v & 3);
            if (key > pos_q) s[v] = -INFINITY;
            mx = fmaxf(mx, s[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        // rows beyond T (t_q >= T) can be fully masked in a tile; keep them finite
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = __expf(m_run - m_use);
        float rs = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = __expf(s[v] - m_use);
            rs += s[v];
        }
        rs += __shfl_xor(rs, 32, 64);
        l_run = l_run * corr + rs;
        m_run = m_new;
#pragma unroll
        for (int j = 0; j < DH / 32; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[j][v] *= corr;
        // O^T += V^T P^T
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = min(k0 + (v >> 2) * 8 + half * 4 + (v & 3), ctx - 1);
            const size_t vat = kv_row_div(a.kv, bt, key, hk) * DH + l32;
#pragma unroll
            for (int j = 0; j < DH / 32; ++j) {
                const float vv = Elem<KT>::to_f32(vp[vat + j * 32]);
                o[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv, s[v], o[j], 0, 0, 0);
            }
        }
    }

    if (t_q >= a.T) return;
    const float inv = 1.0f / l_run;
    OT* op = static_cast<OT*>(a.o) + (static_cast<size_t>(b) * a.T + t_q) * a.hq * DH + h * DH;
#pragma unroll
    for (int j = 0; j < DH / 32; ++j)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int d = j * 32 + vq * 8 + half * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) op[d + i] = Elem<OT>::from_f32(o[j][vq * 4 + i] * inv);
        }
}

// Same algorithm for a half cache on v_mfma_f32_32x32x16_f16: 16 keys or 16 head-dims per
// instruction instead of 2.  K fragments are 16-byte loads (8 consecutive head dims of one
// key); Q is converted to half (already scaled) once; P^T leaves the softmax in registers
// 8m..8m+7 exactly as MFMA m of the PV product wants its B operand (keys 16m + 8b + 4*half
// + i, b < 2, i < 4); V^T is gathered with 2-byte loads for the same keys.
template <typename OT, int DH>
__global__ __launch_bounds__(256) void prefill_attn_f16_kernel(PrefillAttn a, SeqBatch sb) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int qt = gridDim.x - 1 - blockIdx.x;  // longest rows first
    const int h = blockIdx.y * 4 + wave;
    const int b = blockIdx.z;
    if (h >= a.hq) return;
    const int hk = h / (a.hq / a.kv.hkv);
    const int P = sb.pos[b];
    const int32_t* bt = a.kv.block_table + static_cast<size_t>(sb.seq[b]) * a.kv.max_pages;
    const f16_t* __restrict__ kp = static_cast<const f16_t*>(a.kv.k);
    const f16_t* __restrict__ vp = static_cast<const f16_t*>(a.kv.v);
    const int ctx = P + a.T;

    const int t_q = qt * 32 + l32;
    const int t_ld = min(t_q, a.T - 1);
    const size_t qrow = (static_cast<size_t>(b) * a.T + t_ld) * a.hq * DH + h * DH;
    const float scale = 1.0f / sqrtf(static_cast<float>(DH));
    f16x8_t qf[DH / 16];
#pragma unroll
    for (int j = 0; j < DH / 16; ++j) {
        const float4 lo = *reinterpret_cast<const float4*>(a.q + qrow + j * 16 + half * 8);
        const float4 hi = *reinterpret_cast<const float4*>(a.q + qrow + j * 16 + half * 8 + 4);
        qf[j][0] = static_cast<f16_t>(lo.x * scale); qf[j][1] = static_cast<f16_t>(lo.y * scale);
        qf[j][2] = static_cast<f16_t>(lo.z * scale); qf[j][3] = static_cast<f16_t>(lo.w * scale);
        qf[j][4] = static_cast<f16_t>(hi.x * scale); qf[j][5] = static_cast<f16_t>(hi.y * scale);
        qf[j][6] = static_cast<f16_t>(hi.z * scale); qf[j][7] = static_cast<f16_t>(hi.w * scale);
    }
    f32x16 o[DH / 32];
#pragma unroll
    for (int j = 0; j < DH / 32; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[j][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const int pos_q = P + t_q;
    const int last_key = P + min(qt * 32 + 31, a.T - 1);

    for (int k0 = 0; k0 <= last_key; k0 += 32) {
        const int u = min(k0 + l32, ctx - 1);
        const size_t kat = kv_row(a.kv, bt, u, hk) * DH + half * 8;
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int j = 0; j < DH / 16; ++j) {
            const f16x8_t kf = *reinterpret_cast<const f16x8_t*>(kp + kat + j * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[j], s, 0, 0, 0);
        }
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = k0 + (v >> 2) * 8 + half * 4 + (v & 3);
            if (key > pos_q) s[v] = -INFINITY;
            mx = fmaxf(mx, s[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = __expf(m_run - m_use);
        float rs = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = __expf(s[v] - m_use);
            rs += s[v];
        }
        rs += __shfl_xor(rs, 32, 64);
        l_run = l_run * corr + rs;
        m_run = m_new;
#pragma unroll
        for (int j = 0; j < DH / 32; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[j][v] *= corr;
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            f16x8_t pf;
            size_t vat[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                pf[i] = static_cast<f16_t>(s[mm * 8 + i]);
                // register 8*mm + i of this lane is key 16*mm + 8*(i/4) + 4*half + i%4
                const int key = min(k0 + mm * 16 + (i >> 2) * 8 + half * 4 + (i & 3), ctx - 1);
                vat[i] = kv_row(a.kv, bt, key, hk) * DH + l32;
            }
#pragma unroll
            for (int j = 0; j < DH / 32; ++j) {
                f16x8_t vf;
#pragma unroll
                for (int i = 0; i < 8; ++i) vf[i] = vp[vat[i] + j * 32];
                o[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, o[j], 0, 0, 0);
            }
        }
    }

    if (t_q >= a.T) return;
    const float inv = 1.0f / l_run;
    OT* op = static_cast<OT*>(a.o) + (static_cast<size_t>(b) * a.T + t_q) * a.hq * DH + h * DH;
#pragma unroll
    for (int j = 0; j < DH / 32; ++j)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int d = j * 32 + vq * 8 + half * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) op[d + i] = Elem<OT>::from_f32(o[j][vq * 4 + i] * inv);
        }
}

template <typename OT>
static void launch_pa_f16(const PrefillAttn& a, const SeqBatch& sb, hipStream_t st) {
    const dim3 grid((a.T + 31) / 32, (a.hq + 3) / 4, a.B), block(256);
    switch (a.kv.dh) {
        case 32: launch((prefill_attn_f16_kernel<OT, 32>), grid, block, 0, st, a, sb); break;
        case 64: launch((prefill_attn_f16_kernel<OT, 64>), grid, block, 0, st, a, sb); break;
        default: launch((prefill_attn_f16_kernel<OT, 128>), grid, block, 0, st, a, sb); break;
    }
}

template <typename KT, typename OT>
static void launch_pa(const PrefillAttn& a, const SeqBatch& sb, hipStream_t st) {
    const dim3 grid((a.T + 31) / 32, (a.hq + 3) / 4, a.B), block(256);
    switch (a.kv.dh) {
        case 32: launch((prefill_attn_kernel<KT, OT, 32>), grid, block, 0, st, a, sb); break;
        case 64: launch((prefill_attn_kernel<KT, OT, 64>), grid, block, 0, st, a, sb); break;
        default: launch((prefill_attn_kernel<KT, OT, 128>), grid, block, 0, st, a, sb); break;
    }
}

// ---------------------------------------------------------------------------------------
// Prefill attention with key/value tiles staged in LDS (head_dim 64 or 128).
// A workgroup owns 32 QT (128 or 64) consecutive query rows of one (sequence, head): QT waves
// take one 32-row query tile each, and KS groups of such waves split the 32-key blocks between them
// (group g takes blocks g, g + KS, ...), each with its own running max / sum / output, merged
// at the end in group order.  The waves of a group share every K and V tile: the tile is
// fetched once, straight from global memory into a ring of LDS stages (16 bytes per lane,
// addresses from the sequence's block-table row, which is copied to LDS first), the fetch of
// block i + STAGES - 1 in flight while block i is multiplied.  The kernels above instead read
// K and V per wave from global memory and, for V^T, element by element.
// LDS rows are whole K / V rows; 16-byte chunks are XOR-swizzled so that the 16-byte K
// fragment reads (one row per lane) and the element reads of V^T (rows 4 apart in the two
// half-waves) do not collide on banks.
// Same arithmetic as the kernels above: S^T = K Q^T and O^T = V^T P^T on the matrix cores,
// softmax per query column in fp32.
// ---------------------------------------------------------------------------------------
template <typename KT, int DH, int KS, int STAGES, int QT>
__global__ __launch_bounds__(64 * QT * KS) void prefill_attn_lds_kernel(PrefillAttn a, SeqBatch sb) {
    constexpr int QB = 32 * QT;                   // query rows per workgroup
    constexpr bool F16 = sizeof(KT) == 2;
    constexpr int VEC = 16 / sizeof(KT);
    constexpr int CHR = DH / VEC;                 // 16-byte chunks per row
    constexpr int RPI = 64 / CHR;                 // rows per wave-level load
    constexpr int ROWB = DH * sizeof(KT);         // bytes per row
    constexpr int TILE_B = 32 * ROWB;             // one K or V tile
    constexpr int STAGE_B = 2 * TILE_B;
    constexpr int NPER = 2 * 32 / RPI / QT;       // loads per wave per stage
    constexpr int BT_CAP = 2048;                  // block-table entries cached in LDS (the launcher checks the context fits)
    static_assert(CHR >= 8 && (2 * 32 / RPI) % QT == 0, "head_dim 64 or 128");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    int32_t* s_bt = reinterpret_cast<int32_t*>(lds);
    char* ring = lds + BT_CAP * 4;
    const uint32_t ring0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)ring));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave % QT, g = wave / QT;      // query tile in the block, key-split group
    const int l32 = lane & 31, half = lane >> 5;
    const int qg = gridDim.x - 1 - blockIdx.x;    // longest rows first
    const int h = blockIdx.y, b = blockIdx.z;
    const int hk = h / (a.hq / a.kv.hkv);
    const int P = sb.pos[b];
    const int ctx = P + a.T;
    const int32_t* bt = a.kv.block_table + static_cast<size_t>(sb.seq[b]) * a.kv.max_pages;
    const KT* __restrict__ kp = static_cast<const KT*>(a.kv.k);
    const KT* __restrict__ vp = static_cast<const KT*>(a.kv.v);

    // blocks this workgroup walks: up to the diagonal of its last query row
    const int last_row_wg = min(qg * QB + QB - 1, a.T - 1);
    const int nblk_wg = (P + last_row_wg) / 32 + 1;
    const int steps = (nblk_wg + KS - 1) / KS;
    const int npages = (ctx - 1) / a.kv.page + 1;
    for (int i = tid; i < npages; i += 64 * QT * KS) s_bt[i] = bt[i];
    __syncthreads();

    // this lane's share of a stage: NPER loads, each 16 bytes of one K or V row
    auto swz_k = [](int r) { return CHR >= 16 ? (r & 15) : ((r >> 1) & 7); };
    // V rows: consecutive rows land in different 32-byte slots of the row (eight of them when
    // the row has 16 chunks, four when it has 8), so that the column reads of V^T spread over banks
    // (fp32 reads V element by element: there only the two half-waves, rows 4 apart, have to differ)
    auto swz_v = [](int r) { return !F16 ? ((r >> 2) & 1) * 8 : CHR >= 16 ? (r & 7) << 1 : (r & 3) << 1; };
    int ld_row[NPER], ld_chunk[NPER];
    bool ld_isv[NPER];
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
        const int c = wq + QT * i;                // this wave's i-th load of its group's stage
        constexpr int PER_TILE = 32 / RPI;
        ld_isv[i] = c >= PER_TILE;
        const int cc = ld_isv[i] ? c - PER_TILE : c;
        ld_row[i] = cc * RPI + lane / CHR;
        ld_chunk[i] = (lane % CHR) ^ (ld_isv[i] ? swz_v(ld_row[i]) : swz_k(ld_row[i]));
    }
    auto issue = [&](int step) {                  // block (step * KS + g) -> stage step % STAGES of group g
        int kb = step * KS + g;
        if (kb >= nblk_wg) kb = nblk_wg - 1;      // past the end: a harmless reload
        const uint32_t st0 = ring0 + (static_cast<uint32_t>(g) * STAGES + step % STAGES) * STAGE_B;
#pragma unroll
        for (int i = 0; i < NPER; ++i) {
            const int u = min(kb * 32 + ld_row[i], ctx - 1);
            int pg, slot;
            kv_split(a.kv, u, &pg, &slot);
            const size_t row = (static_cast<size_t>(s_bt[pg]) * a.kv.hkv + hk) * a.kv.page + slot;
            const KT* src = (ld_isv[i] ? vp : kp) + row * DH + ld_chunk[i] * VEC;
            const int c = wq + QT * i;
            lds_dma16(src, st0 + (ld_isv[i] ? TILE_B : 0) + (ld_isv[i] ? c - 32 / RPI : c) * 1024);
        }
    };

    // query fragments (scaled), this wave's 32 rows
    const int t_q = qg * QB + wq * 32 + l32;
    const int t_ld = min(t_q, a.T - 1);
    const size_t qrow = (static_cast<size_t>(b) * a.T + t_ld) * a.hq * DH + h * DH;
    const float scale = 1.0f / sqrtf(static_cast<float>(DH));
    float4 qf[DH / 8];                            // fp32: 4 floats per k-group of 8; half: 8 halfs per k-group of 16
    if constexpr (F16) {
#pragma unroll
        for (int j = 0; j < DH / 16; ++j) {
            const float4 lo = *reinterpret_cast<const float4*>(a.q + qrow + j * 16 + half * 8);
            const float4 hi = *reinterpret_cast<const float4*>(a.q + qrow + j * 16 + half * 8 + 4);
            f16x8_t t;
            t[0] = static_cast<f16_t>(lo.x * scale); t[1] = static_cast<f16_t>(lo.y * scale);
            t[2] = static_cast<f16_t>(lo.z * scale); t[3] = static_cast<f16_t>(lo.w * scale);
            t[4] = static_cast<f16_t>(hi.x * scale); t[5] = static_cast<f16_t>(hi.y * scale);
            t[6] = static_cast<f16_t>(hi.z * scale); t[7] = static_cast<f16_t>(hi.w * scale);
            qf[j] = __builtin_bit_cast(float4, t);
        }
    } else {
#pragma unroll
        for (int j = 0; j < DH / 8; ++j) {
            qf[j] = *reinterpret_cast<const float4*>(a.q + qrow + j * 8 + half * 4);
            qf[j].x *= scale; qf[j].y *= scale; qf[j].z *= scale; qf[j].w *= scale;
        }
    }
    f32x16 o[DH / 32];
#pragma unroll
    for (int j = 0; j < DH / 32; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[j][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const int pos_q = P + t_q;
    // diagonal of this wave's tile; a tile that starts past the last row has nothing to do
    const int last_key = qg * QB + wq * 32 < a.T ? P + min(qg * QB + wq * 32 + 31, a.T - 1) : -1;

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s);
    for (int step = 0; step < steps; ++step) {
        wait_vmcnt<NPER*(STAGES - 2)>();
        __syncthreads();
        issue(step + STAGES - 1);
        const int k0 = (step * KS + g) * 32;
        if (k0 > last_key) continue;              // above this wave's diagonal (it still fetched and synchronised)
        const char* sK = ring + (g * STAGES + step % STAGES) * STAGE_B;
        const char* sV = sK + TILE_B;
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
        if constexpr (F16) {
#pragma unroll
            for (int j = 0; j < DH / 16; ++j) {
                const float4 kf = *reinterpret_cast<const float4*>(sK + l32 * ROWB + (((j * 2 + half) ^ swz_k(l32)) << 4));
                s = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, kf), __builtin_bit_cast(f16x8_t, qf[j]), s, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < DH / 8; ++j) {
                const float4 kf = *reinterpret_cast<const float4*>(sK + l32 * ROWB + (((j * 2 + half) ^ swz_k(l32)) << 4));
                s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.x, qf[j].x, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.y, qf[j].y, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.z, qf[j].z, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.w, qf[j].w, s, 0, 0, 0);
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = k0 + (v >> 2) * 8 + half * 4 + (v & 3);
            if (key > pos_q) s[v] = -INFINITY;
            mx = fmaxf(mx, s[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = __expf(m_run - m_use);
        float rs = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = __expf(s[v] - m_use);
            rs += s[v];
        }
        rs += __shfl_xor(rs, 32, 64);
        l_run = l_run * corr + rs;
        m_run = m_new;
#pragma unroll
        for (int j = 0; j < DH / 32; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[j][v] *= corr;
        // O^T += V^T P^T; register v of a lane is key (v/4)*8 + 4*half + v%4 of the block
        if constexpr (F16) {
#pragma unroll
            for (int mm = 0; mm < 2; ++mm) {
                f16x8_t pf;
#pragma unroll
                for (int i = 0; i < 8; ++i) pf[i] = static_cast<f16_t>(s[mm * 8 + i]);
#pragma unroll
                for (int j = 0; j < DH / 32; ++j) {
                    // V^T fragment by two transposing LDS reads (ds_read_b64_tr_b16): within
                    // 16 lanes, lane m hands in the address of 4 halfs of one row and lane
                    // (g, e) = (m / 4, m % 4) receives element e of the rows of lanes g, g + 4,
                    // g + 8, g + 12.  Lane m therefore points at key row m / 4 of the group,
                    // features 4 * (m % 4) .. + 3 of its 16-feature block, and gets the four
                    // keys of the group for its own feature.
                    typedef short i16x4_t __attribute__((ext_vector_type(4)));
                    typedef short i16x8_t __attribute__((ext_vector_type(8)));
                    i16x8_t vraw;
#pragma unroll
                    for (int grp = 0; grp < 2; ++grp) {
                        const int m16 = lane & 15, dblk = (lane >> 4) & 1;
                        const int r = mm * 16 + grp * 8 + half * 4 + (m16 >> 2);
                        const int d = j * 32 + dblk * 16 + 4 * (m16 & 3);
                        const char* at = sV + r * ROWB + (((d >> 3) ^ swz_v(r)) << 4) + (d & 7) * 2;
                        const i16x4_t t = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) i16x4_t*)(at));
                        vraw[grp * 4 + 0] = t[0]; vraw[grp * 4 + 1] = t[1]; vraw[grp * 4 + 2] = t[2]; vraw[grp * 4 + 3] = t[3];
                    }
                    o[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, vraw), pf, o[j], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = (v >> 2) * 8 + half * 4 + (v & 3);
#pragma unroll
                for (int j = 0; j < DH / 32; ++j) {
                    const int d = j * 32 + l32;
                    const float vv = *reinterpret_cast<const float*>(sV + r * ROWB + (((d >> 2) ^ swz_v(r)) << 4) + (d & 3) * 4);
                    o[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv, s[v], o[j], 0, 0, 0);
                }
            }
        }
    }
    wait_vmcnt<0>();

    // merge the key-split groups in group order (group 0 holds the result)
    if constexpr (KS > 1) {
        __syncthreads();                          // every wave is done with the ring
        float* xo = reinterpret_cast<float*>(ring);                    // [QT][DH/32*16][64]
        float* xm = xo + QT * (DH / 32 * 16) * 64;                     // [QT][2][64]
        for (int src = 1; src < KS; ++src) {
            if (g == src) {
#pragma unroll
                for (int j = 0; j < DH / 32; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) xo[(wq * (DH / 32 * 16) + j * 16 + v) * 64 + lane] = o[j][v];
                xm[(wq * 2 + 0) * 64 + lane] = m_run;
                xm[(wq * 2 + 1) * 64 + lane] = l_run;
            }
            __syncthreads();
            if (g == 0) {
                const float m2 = xm[(wq * 2 + 0) * 64 + lane], l2 = xm[(wq * 2 + 1) * 64 + lane];
                const float m_new = fmaxf(m_run, m2);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                const float c1 = __expf(m_run - m_use), c2 = __expf(m2 - m_use);
                l_run = l_run * c1 + l2 * c2;
                m_run = m_new;
#pragma unroll
                for (int j = 0; j < DH / 32; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        o[j][v] = o[j][v] * c1 + xo[(wq * (DH / 32 * 16) + j * 16 + v) * 64 + lane] * c2;
            }
            __syncthreads();
        }
    }
    if (g != 0 || t_q >= a.T) return;
    const float inv = 1.0f / l_run;
    typedef typename ActOf<KT>::type OT;
    OT* op = static_cast<OT*>(a.o) + (static_cast<size_t>(b) * a.T + t_q) * a.hq * DH + h * DH;
#pragma unroll
    for (int j = 0; j < DH / 32; ++j)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int d = j * 32 + vq * 8 + half * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) op[d + i] = Elem<OT>::from_f32(o[j][vq * 4 + i] * inv);
        }
}

template <typename KT, int DH, int KS, int STAGES, int QT>
static void launch_pa_lds_q(const PrefillAttn& a, const SeqBatch& sb, hipStream_t st) {
    constexpr size_t lds = 2048 * 4 + static_cast<size_t>(KS) * STAGES * 2 * 32 * DH * sizeof(KT);
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    static_assert(KS == 1 || static_cast<size_t>(KS) * STAGES * 2 * 32 * DH * sizeof(KT) >= QT * (DH / 32 * 16 + 2) * 64 * 4,
                  "the merge buffer lives in the ring");
    static std::once_flag once;  // more than 64 KB of LDS per workgroup is an opt-in
    std::call_once(once, [] {
        note_kernel_attribute(hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_attn_lds_kernel<KT, DH, KS, STAGES, QT>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    });
    const dim3 grid((a.T + 32 * QT - 1) / (32 * QT), a.hq, a.B);
    launch(prefill_attn_lds_kernel<KT, DH, KS, STAGES, QT>, grid, dim3(64 * QT * KS), lds, st, a, sb);
}

// Query rows per workgroup: 128, or 64 when 128-row blocks would not even give every compute
// unit a workgroup (7B shape, 512 tokens, one sequence: 128 workgroups; 64-row blocks make it
// 256 and the fp32 kernel 82 -> 58 us).  With a workgroup per unit already, the smaller blocks'
// lower K/V reuse costs more than the better balance of the causal triangle gains (half
// precision, 1024 tokens: 43 -> 72 us).
template <typename KT, int DH, int KS, int STAGES>
static void launch_pa_lds(const PrefillAttn& a, const SeqBatch& sb, hipStream_t st) {
    const long wgs128 = static_cast<long>((a.T + 127) / 128) * a.hq * a.B;
    if (wgs128 < 256) launch_pa_lds_q<KT, DH, KS, STAGES, 2>(a, sb, st);
    else launch_pa_lds_q<KT, DH, KS, STAGES, 4>(a, sb, st);
}

void launch_prefill_attn(const PrefillAttn& a, const SeqBatch& sb, hipStream_t st) {
    // LDS-staged kernel for the usual head sizes (activations and cache of one type), as long
    // as every sequence's block-table row fits the kernel's LDS copy
    int max_ctx = 0;
    for (int b = 0; b < sb.n; ++b) max_ctx = max_ctx > sb.pos[b] + a.T ? max_ctx : sb.pos[b] + a.T;
    const bool fits = (max_ctx - 1) / a.kv.page + 1 <= 2048;
    if (!fits) {
    } else if (a.kv_dtype == DT_F32 && a.out_dtype == DT_F32) {
        if (a.kv.dh == 128) return launch_pa_lds<float, 128, 2, 2>(a, sb, st);
        if (a.kv.dh == 64) return launch_pa_lds<float, 64, 2, 3>(a, sb, st);
    }
    else if (a.kv_dtype != DT_F32 && a.out_dtype != DT_F32) {
        if (a.kv.dh == 128) return launch_pa_lds<f16_t, 128, 2, 3>(a, sb, st);
        if (a.kv.dh == 64) return launch_pa_lds<f16_t, 64, 2, 3>(a, sb, st);
    }
    if (a.kv_dtype == DT_F32) {
        if (a.out_dtype == DT_F32) launch_pa<float, float>(a, sb, st);
        else launch_pa<float, f16_t>(a, sb, st);
    } else {
        if (a.out_dtype == DT_F32) launch_pa_f16<float>(a, sb, st);
        else launch_pa_f16<f16_t>(a, sb, st);
    }
}

}  // namespace shk
