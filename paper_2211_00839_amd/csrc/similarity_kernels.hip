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
template <typename T, bool FAST>
__device__ __forceinline__ void gram_mainloop(const T *__restrict__ X, long long ldx, int d, bool vec_ok,
                                              const int (&arow)[4], const int (&brow)[2],
                                              unsigned char *__restrict__ lds, f32x16 (&acc)[4][2])
{
    constexpr int BK = Elem<T>::BK;
    constexpr int EPC = CHUNK / (int)sizeof(T);   // elements per chunk
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

    uint4 ra[4], rb[2];
#pragma unroll
    for (int u = 0; u < 4; ++u) ra[u] = load_chunk<T, FAST>(X, ldx, arow[u], cpart * EPC, d, vec_ok);
#pragma unroll
    for (int u = 0; u < 2; ++u) rb[u] = load_chunk<T, FAST>(X, ldx, brow[u], cpart * EPC, d, vec_ok);
#pragma unroll
    for (int u = 0; u < 4; ++u)
        *reinterpret_cast<uint4 *>(lds + (crow0 + 64 * u) * ROWP + cpart * CHUNK) = ra[u];
#pragma unroll
    for (int u = 0; u < 2; ++u)
        *reinterpret_cast<uint4 *>(lds + A_BYTES + (crow0 + 64 * u) * ROWP + cpart * CHUNK) = rb[u];
    __syncthreads();

    // lanes 0-31 take the first 16 bytes of each 32-byte k group, lanes 32-63 the second
    const int koff = (lane >> 5) * CHUNK;
    const int a_base = (wr * 128 + (lane & 31)) * ROWP + koff;
    const int b_base = A_BYTES + (wc * 64 + (lane & 31)) * ROWP + koff;

    int stage = 0;
    for (int k0 = 0; k0 < d; k0 += BK) {
        const bool more = k0 + BK < d;
        if (more) {
#pragma unroll
            for (int u = 0; u < 4; ++u) ra[u] = load_chunk<T, FAST>(X, ldx, arow[u], k0 + BK + cpart * EPC, d, vec_ok);
#pragma unroll
            for (int u = 0; u < 2; ++u) rb[u] = load_chunk<T, FAST>(X, ldx, brow[u], k0 + BK + cpart * EPC, d, vec_ok);
        }
        const unsigned char *cur = lds + stage * STAGE_BYTES;
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
        if (more) {
            unsigned char *nxt = lds + (stage ^ 1) * STAGE_BYTES;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                *reinterpret_cast<uint4 *>(nxt + (crow0 + 64 * u) * ROWP + cpart * CHUNK) = ra[u];
#pragma unroll
            for (int u = 0; u < 2; ++u)
                *reinterpret_cast<uint4 *>(nxt + A_BYTES + (crow0 + 64 * u) * ROWP + cpart * CHUNK) = rb[u];
        }
        __syncthreads();
        stage ^= 1;
    }
}

// Gram tile + Gaussian epilogue.  grid = (column tiles, row tiles).
template <typename T, bool FAST>
__global__ void __launch_bounds__(THREADS, 2)
k_gram_rbf(const T *__restrict__ X, long long ldx, const int32_t *__restrict__ row_index, int n, int d,
           const float *__restrict__ sq, float exp_scale, float *__restrict__ S, long long lds_out,
           int ncols_pad)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE_BYTES];

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

    f32x16 acc[4][2];
    gram_mainloop<T, FAST>(X, ldx, d, vec_ok, arow, brow, lds, acc);

    // epilogue: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane>>5) + (r&3)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int j = j0 + wc * 64 + b * 32 + (lane & 31);
        const float sqj = j < n ? sq[j] : 0.f;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wr * 128 + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (i < n && j < ncols_pad) {
                    float s = 0.f;
                    if (j < n) {
                        float dist = sq[i] + sqj - 2.f * acc[a][b][r];
                        dist = fmaxf(dist, 0.f);
                        s = (i == j) ? 1.f : exp2f(dist * exp_scale);
                    }
                    S[(size_t)i * lds_out + j] = s;
                }
            }
        }
    }
}

} // namespace sim
