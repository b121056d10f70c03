// Similarity build for gfx950: S = exp(-(|x_i|^2 + |x_j|^2 - 2 x_i.x_j) / (2 sigma^2)),
// the Gaussian kernel on the L2 distance of Section 4 (arXiv 2211.00839), with the
// Gram matrix X X^T on the matrix cores (fp32 accumulation) and the kernel fused
// into the epilogue.  S(i,j) and S(j,i) go through the same products in the same
// order, so the result is symmetric bit for bit; the diagonal is forced to 1.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sim {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 256;          // tile rows (x_i)
constexpr int BN = 128;          // tile columns (x_j)
constexpr int CHUNK = 16;        // bytes per global->LDS chunk
constexpr int ROWB = 64;         // bytes of k per tile row and stage
constexpr int ROWP = 80;         // padded LDS row pitch in bytes (spreads the banks)
constexpr int THREADS = 256;
constexpr int A_BYTES = BM * ROWP;
constexpr int B_BYTES = BN * ROWP;
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;   // 30 KB; two stages per workgroup

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int BK = 16; };
template <> struct Elem<__bf16> { static constexpr int BK = 32; };

// 2^x by the hardware instruction (about 1 ulp); results below 2^-126 flush to 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// The similarity from the Gram value g = x_i . x_j and the pre-scaled norms
// sq_s = |x|^2 * c, c = -log2(e) / (2 sigma^2):  2^min(0, sq_i_s + sq_j_s - 2 c g).
// Every kernel that needs a similarity goes through this one expression, so that
// S(i,j) is the same bits wherever it is computed.
__device__ __forceinline__ float rbf_value(float gram, float sqi_s, float sqj_s, float scale2)
{
    return fast_exp2(fminf(fmaf(gram, scale2, sqi_s + sqj_s), 0.f));
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }

// One 16-byte chunk of row `row`, k range [k, k + 16/sizeof(T)), zero beyond d.
// FAST: rows are 16-byte aligned and d is a multiple of the stage depth, so every
// chunk is one aligned vector load and the main loop carries no branches.
template <typename T, bool FAST>
__device__ __forceinline__ uint4 load_chunk(const T *__restrict__ X, long long ldx, int row, int k, int d,
                                            bool vec_ok)
{
    constexpr int E = CHUNK / (int)sizeof(T);
    const T *p = X + (size_t)row * ldx + k;
    if constexpr (FAST) return *reinterpret_cast<const uint4 *>(p);
    if (vec_ok && k + E <= d) return *reinterpret_cast<const uint4 *>(p);
    union { uint4 u; T e[E]; } tmp;
    tmp.u = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < E; ++i)
        if (k + i < d) tmp.e[i] = p[i];
    return tmp.u;
}

// Squared row norms, double accumulation, fixed order: one wave per row.
template <typename T>
__global__ void __launch_bounds__(256)
k_row_norms(const T *__restrict__ X, long long ldx, const int32_t *__restrict__ row_index, int n, int d,
            float *__restrict__ sq)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const int r = row_index ? row_index[i] : i;
    const T *p = X + (size_t)r * ldx;
    double a = 0.0;
    for (int t = lane; t < d; t += 64) {
        const double v = (double)to_f32(p[t]);
        a += v * v;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);
    if (lane == 0) sq[i] = (float)a;
}

// ---------------------------------------------------------------------------
// Gram main loop of one 256 x 128 tile: acc += X[arow] . X[brow]^T over all of d.
// 4 waves as 2 x 2; a wave owns 128 x 64 = 4 x 2 MFMA 32x32 tiles (a 4x2 wave
// tile needs 0.75 KB of LDS reads per MFMA, which the LDS can feed at the full
// MFMA rate; a 2x2 one cannot).  k advances 64 bytes per row and stage (32 bf16
// or 16 fp32); stages are double-buffered in LDS, one barrier each: while a
// stage is multiplied the next one is already in registers on its way to LDS.
// arow[u], brow[u]: rows of X behind the 16-byte chunks this thread stages.
// ---------------------------------------------------------------------------
// Multiply one LDS stage into the accumulators (two k sub-steps of 32 bytes).
template <typename T>
__device__ __forceinline__ void gram_stage_mma(const unsigned char *__restrict__ cur, int a_base, int b_base,
                                               f32x16 (&acc)[4][2])
{
#pragma unroll
    for (int kk = 0; kk < ROWB / 32; ++kk) {
        uint4 fa[4], fb[2];
#pragma unroll
        for (int m = 0; m < 4; ++m) fa[m] = *reinterpret_cast<const uint4 *>(cur + a_base + m * 32 * ROWP + kk * 32);
#pragma unroll
        for (int m = 0; m < 2; ++m) fb[m] = *reinterpret_cast<const uint4 *>(cur + b_base + m * 32 * ROWP + kk * 32);
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, fa[a]), __builtin_bit_cast(bf16x8, fb[b]), acc[a][b], 0, 0, 0);
        } else {
            // four 32x32x2 products; lanes<32 carry k = e, lanes>=32 carry k = 4+e,
            // for both operands alike, so every k of the group is used exactly once
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        const f32x4 va = __builtin_bit_cast(f32x4, fa[a]);
                        const f32x4 vb = __builtin_bit_cast(f32x4, fb[b]);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], vb[e], acc[a][b], 0, 0, 0);
                    }
        }
    }
}

// The main loop.  Global loads run NPRE stages ahead of the multiply (a stage
// is only ~0.2 us of MFMA work, far less than a trip to L2 or HBM): NPRE
// register sets hold the stages in flight, the oldest is written to the free LDS
// buffer right after the multiply of the current stage, then its registers are
// reloaded with the stage NPRE ahead.
template <typename T, bool FAST>
__device__ __forceinline__ void gram_mainloop(const T *__restrict__ X, long long ldx, int d, bool vec_ok,
                                              const int (&arow)[4], const int (&brow)[2],
                                              unsigned char *__restrict__ lds, f32x16 (&acc)[4][2])
{
    constexpr int BK = Elem<T>::BK;
    constexpr int EPC = CHUNK / (int)sizeof(T);   // elements per chunk
    constexpr int NPRE = 1;   // generic path only: unaligned rows or ragged d; the aligned case uses gram_mainloop_dma
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int cpart = tid & 3;                    // which 16 bytes of the row's 64
    const int crow0 = tid >> 2;                   // rows crow0 + 64 u

#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int nstage = (d + BK - 1) / BK;
    uint4 ra[NPRE][4], rb[NPRE][2];
    auto load_stage = [&](int set, int stage) {
        const int k = stage * BK + cpart * EPC;
#pragma unroll
        for (int u = 0; u < 4; ++u) ra[set][u] = load_chunk<T, FAST>(X, ldx, arow[u], k, d, vec_ok);
#pragma unroll
        for (int u = 0; u < 2; ++u) rb[set][u] = load_chunk<T, FAST>(X, ldx, brow[u], k, d, vec_ok);
    };
    auto store_stage = [&](int set, unsigned char *dst) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            *reinterpret_cast<uint4 *>(dst + (crow0 + 64 * u) * ROWP + cpart * CHUNK) = ra[set][u];
#pragma unroll
        for (int u = 0; u < 2; ++u)
            *reinterpret_cast<uint4 *>(dst + A_BYTES + (crow0 + 64 * u) * ROWP + cpart * CHUNK) = rb[set][u];
    };

    // prologue: stage 0 goes straight to LDS, stages 1..NPRE stay in flight in registers
    load_stage(0, 0);
    store_stage(0, lds);
#pragma unroll
    for (int i = 0; i < NPRE; ++i)
        if (1 + i < nstage) load_stage(i, 1 + i);
    __syncthreads();

    // lanes 0-31 take the first 16 bytes of each 32-byte k group, lanes 32-63 the second
    const int koff = (lane >> 5) * CHUNK;
    const int a_base = (wr * 128 + (lane & 31)) * ROWP + koff;
    const int b_base = A_BYTES + (wc * 64 + (lane & 31)) * ROWP + koff;

    // iteration s: LDS[s&1] holds stage s; register set (s % NPRE) holds stage s+1.
    // Unrolled by 2*NPRE so that register sets and LDS buffers are addressed
    // statically; the steady-state loop carries no conditions (every stage it
    // touches exists), the last stages run through the guarded tail.
    constexpr int UNR = 2 * NPRE;
    int s0 = 0;
    for (; s0 + UNR + NPRE < nstage; s0 += UNR) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            gram_stage_mma<T>(lds + (i & 1) * STAGE_BYTES, a_base, b_base, acc);
            store_stage(i % NPRE, lds + ((i + 1) & 1) * STAGE_BYTES);
            load_stage(i % NPRE, s0 + i + 1 + NPRE);
            __syncthreads();
        }
    }
    // s0 is a multiple of UNR (even), so buffer and register-set parities carry over
#pragma unroll 1
    for (; s0 < nstage; s0 += NPRE) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i) {
            const int s = s0 + i;
            if (s < nstage) {
                gram_stage_mma<T>(lds + (s & 1) * STAGE_BYTES, a_base, b_base, acc);
                if (s + 1 < nstage) store_stage(i, lds + ((s + 1) & 1) * STAGE_BYTES);
                if (s + 1 + NPRE < nstage) load_stage(i, s + 1 + NPRE);
                __syncthreads();
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Fast main loop (rows 16-byte aligned, d a multiple of the stage depth): the
// stages go from global memory straight into LDS (global_load_lds_dwordx4: lane
// L of a wave drops its 16 bytes at LDS base + 16 L), three stages deep, no
// registers and no ds_write in between.  Rows are 64 bytes in LDS, unpadded;
// the 16-byte chunk c of row r sits at chunk position c ^ swizzle(r), which
// keeps both 8- and 16-lane groups of a ds_read_b128 on distinct banks.  The
// loads are issued from inline asm so that their completion is awaited by
// explicit vmcnt counts (stage s must have landed, younger stages may fly); the
// compiler would otherwise wait for all of them at every barrier.
// ---------------------------------------------------------------------------
constexpr int DMA_STAGES = 3;
constexpr int DMA_STAGE_BYTES = (BM + BN) * ROWB;      // 24 KB
constexpr int DMA_LDS_BYTES = DMA_STAGES * DMA_STAGE_BYTES;

__device__ __forceinline__ int lds_swizzle(int row)
{
    return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
}

__device__ __forceinline__ void dma16(const void *gptr, unsigned lds_addr)
{
    unsigned saved;
    asm volatile("s_mov_b32 %0, m0\n\t"
                 "s_mov_b32 m0, %2\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, off\n\t"
                 "s_mov_b32 m0, %0"
                 : "=&s"(saved)
                 : "v"(gptr), "s"(lds_addr)
                 : "memory");
}

// Tile row (0..255 = A rows, 256..383 = B rows) and k chunk that lane `lane` of
// wave `wave` fetches with its u-th load of a stage.
__device__ __forceinline__ void dma_slot(int wave, int u, int lane, int *tile_row, int *chunk)
{
    const int row = (wave * 6 + u) * 16 + (lane >> 2);
    *tile_row = row;
    *chunk = (lane & 3) ^ lds_swizzle(row);
}

// gp[u]: address of this lane's chunk of stage 0 for its u-th load (see dma_slot).
template <typename T>
__device__ __forceinline__ void gram_mainloop_dma(const T *const (&gp)[6], int d, unsigned char *lds,
                                                  f32x16 (&acc)[4][2])
{
    constexpr int BK = Elem<T>::BK;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;
    auto issue = [&](int stage, int buf) {
#pragma unroll
        for (int u = 0; u < 6; ++u)
            dma16(gp[u] + (size_t)stage * BK, lds_base + buf * DMA_STAGE_BYTES + (wave * 6 + u) * 1024);
    };
    // fragment addresses inside a stage: lanes 0-31 take k chunk 2 kk, lanes 32-63 chunk 2 kk + 1
    const int hi = lane >> 5;
    int aoff[4][2], boff[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int row = wr * 128 + 32 * m + (lane & 31);
            aoff[m][kk] = row * ROWB + (((kk * 2 + hi) ^ lds_swizzle(row)) << 4);
        }
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int row = BM + wc * 64 + 32 * m + (lane & 31);
            boff[m][kk] = row * ROWB + (((kk * 2 + hi) ^ lds_swizzle(row)) << 4);
        }
    }
    auto mma = [&](const unsigned char *cur) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            uint4 fa[4], fb[2];
#pragma unroll
            for (int m = 0; m < 4; ++m) fa[m] = *reinterpret_cast<const uint4 *>(cur + aoff[m][kk]);
#pragma unroll
            for (int m = 0; m < 2; ++m) fb[m] = *reinterpret_cast<const uint4 *>(cur + boff[m][kk]);
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, fa[a]), __builtin_bit_cast(bf16x8, fb[b]), acc[a][b], 0, 0, 0);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int a = 0; a < 4; ++a)
#pragma unroll
                        for (int b = 0; b < 2; ++b) {
                            const f32x4 va = __builtin_bit_cast(f32x4, fa[a]);
                            const f32x4 vb = __builtin_bit_cast(f32x4, fb[b]);
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], vb[e], acc[a][b], 0, 0, 0);
                        }
            }
        }
    };

    const int nstage = d / BK;
    issue(0, 0);
    if (nstage > 1) issue(1, 1);
    int s = 0;
    // Before the barrier of iteration s this wave's loads of stage s have landed (the 6
    // loads of stage s+1 may still fly); after it everyone's have, and everyone is done
    // reading the buffer that stage s+2 is about to overwrite.
    for (; s + 2 < nstage; ++s) {
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        issue(s + 2, (s + 2) % DMA_STAGES);
        mma(lds + (s % DMA_STAGES) * DMA_STAGE_BYTES);
    }
    for (; s < nstage; ++s) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        mma(lds + (s % DMA_STAGES) * DMA_STAGE_BYTES);
    }
    __builtin_amdgcn_s_barrier();   // everyone is done with the ring
}

// Gram tile + Gaussian epilogue.  grid = (column tiles, row tiles).
template <typename T, bool FAST>
__global__ void __launch_bounds__(THREADS, 2)
k_gram_rbf(const T *__restrict__ X, long long ldx, const int32_t *__restrict__ row_index, int n, int d,
           const float *__restrict__ sq, float exp_scale, float *__restrict__ S, long long lds_out,
           int ncols_pad)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[FAST ? DMA_LDS_BYTES : 2 * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BN;

    if (j0 >= n) {
        // tile entirely in the zero padding of the output pitch
        for (int e = tid; e < BM * BN; e += THREADS) {
            const int i = i0 + e / BN, j = j0 + e % BN;
            if (i < n && j < ncols_pad) S[(size_t)i * lds_out + j] = 0.f;
        }
        return;
    }

    f32x16 acc[4][2];
    if constexpr (FAST) {
        const T *gp[6];
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            int trow, chunk;
            dma_slot(wave, u, lane, &trow, &chunk);
            const int gi = trow < BM ? min(i0 + trow, n - 1) : min(j0 + trow - BM, n - 1);
            const int row = row_index ? row_index[gi] : gi;
            gp[u] = X + (size_t)row * ldx + chunk * (CHUNK / (int)sizeof(T));
        }
        gram_mainloop_dma<T>(gp, d, lds, acc);
    } else {
        const bool vec_ok = ((reinterpret_cast<uintptr_t>(X) & 15) == 0) && ((ldx * (long long)sizeof(T)) % 16 == 0);
        int arow[4], brow[2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ai = min(i0 + (tid >> 2) + 64 * u, n - 1);
            arow[u] = row_index ? row_index[ai] : ai;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int bj = min(j0 + (tid >> 2) + 64 * u, n - 1);
            brow[u] = row_index ? row_index[bj] : bj;
        }
        gram_mainloop<T, false>(X, ldx, d, vec_ok, arow, brow, lds, acc);
    }

    // epilogue: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane>>5) + (r&3).
    // The row norms, pre-multiplied by the (negative) exponent scale, go through LDS.
    float *sq_rows = reinterpret_cast<float *>(lds);     // the stage ring is idle now
    {
        const int i = i0 + tid;
        sq_rows[tid] = i < n ? sq[i] * exp_scale : 0.f;
    }
    __syncthreads();
    const float scale2 = -2.f * exp_scale;
    const bool interior = i0 + BM <= n && j0 + BN <= n;
    const bool on_diagonal = i0 < j0 + BN && j0 < i0 + BM;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int j = j0 + wc * 64 + b * 32 + (lane & 31);
        const float sqj = j < n ? sq[j] * exp_scale : 0.f;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int rl = wr * 128 + a * 32 + rq * 8 + (lane >> 5) * 4;     // 4 consecutive rows
                const float4 sqi4 = *reinterpret_cast<const float4 *>(sq_rows + rl);
                const float sqi[4] = {sqi4.x, sqi4.y, sqi4.z, sqi4.w};
                float *dst = S + (size_t)(i0 + rl) * lds_out + j;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = i0 + rl + e;
                    float v = rbf_value(acc[a][b][rq * 4 + e], sqi[e], sqj, scale2);
                    if (on_diagonal && i == j) v = 1.f;
                    if (interior) {
                        dst[(size_t)e * lds_out] = v;
                    } else if (i < n && j < ncols_pad) {
                        dst[(size_t)e * lds_out] = j < n ? v : 0.f;
                    }
                }
            }
        }
    }
}

} // namespace sim
