// Similarity build for gfx950: S = exp(-(|x_i|^2 + |x_j|^2 - 2 x_i.x_j) / (2 sigma^2)),
// the Gaussian kernel on the L2 distance of Section 4 (arXiv 2211.00839), with the
// Gram matrix X X^T on the matrix cores (fp32 accumulation) and the kernel fused
// into the epilogue.  S(i,j) and S(j,i) go through the same products in the same
// order, so the result is symmetric bit for bit; the diagonal is forced to 1.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

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
// sq_s = |x|^2 * c, c = -log2(e) / (2 sigma^2):  min(1, 2^(sq_i_s + sq_j_s - 2 c g)),
// the min being the clamp-to-[0,1] output modifier of the exponential instruction.
// Every kernel that needs a similarity goes through this one expression, so that
// S(i,j) is the same bits wherever it is computed.
__device__ __forceinline__ float rbf_value(float gram, float sqi_s, float sqj_s, float scale2)
{
    return __builtin_amdgcn_fmed3f(fast_exp2(fmaf(gram, scale2, sqi_s + sqj_s)), 0.f, 1.f);
}

enum { EPI_RBF = 0, EPI_DISTANCE = 1, EPI_RBF_MIRROR = 2 };

// The L2 distance from the Gram value and the two squared norms, clamped at 0 before the root
// (the hardware root, about 1 ulp; squared distances here are far from the denormal range or 0).
__device__ __forceinline__ float distance_value(float gram, float sqi, float sqj)
{
    return __builtin_amdgcn_sqrtf(fmaxf(fmaf(gram, -2.f, sqi + sqj), 0.f));
}

// Sum of one tile's distances over its 256 threads in a fixed order (lanes by butterfly, then the
// four waves in order); thread 0 stores it.  `scratch`: 4 doubles of LDS nobody else is using.
__device__ __forceinline__ void tile_distance_sum(double mine, double *scratch, int tid, double *out)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off);
    if ((tid & 63) == 0) scratch[tid >> 6] = mine;
    __syncthreads();
    if (tid == 0) *out = ((scratch[0] + scratch[1]) + scratch[2]) + scratch[3];
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }

// One 16-byte chunk of row `row`, k range [k, k + 16/sizeof(T)), zero beyond d.
template <typename T>
__device__ __forceinline__ uint4 load_chunk(const T *__restrict__ X, long long ldx, int row, int k, int d,
                                            bool vec_ok)
{
    constexpr int E = CHUNK / (int)sizeof(T);
    const T *p = X + (size_t)row * ldx + k;
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
// General path.  Gram main loop of one 256 x 128 tile: acc += X[arow] . X[brow]^T over all of d.
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
template <typename T>
__device__ __forceinline__ void gram_mainloop(const T *__restrict__ X, long long ldx, int d, bool vec_ok,
                                              const int (&arow)[4], const int (&brow)[2],
                                              unsigned char *__restrict__ lds, f32x16 (&acc)[4][2])
{
    constexpr int BK = Elem<T>::BK;
    constexpr int EPC = CHUNK / (int)sizeof(T);   // elements per chunk
    constexpr int NPRE = 1;   // general path only: unaligned rows or ragged d; the aligned case uses pipe::Pipe
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
        for (int u = 0; u < 4; ++u) ra[set][u] = load_chunk<T>(X, ldx, arow[u], k, d, vec_ok);
#pragma unroll
        for (int u = 0; u < 2; ++u) rb[set][u] = load_chunk<T>(X, ldx, brow[u], k, d, vec_ok);
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
// Fast path (rows 16-byte aligned, row length a multiple of 128 bytes): a 256 x 256
// tile per 256-thread workgroup, 4 waves as 2 x 2, each wave 4 x 4 MFMA 32x32
// tiles (the 256 accumulator registers of a lane fill the AGPR file, one wave per
// SIMD).  Per unit of k the tile reads 512 feature rows for 65 536 multiply-adds,
// the least traffic between L2 and the compute unit a single workgroup can have.
//
// The features go from global memory straight into LDS (global_load_lds_dwordx4:
// lane L of a wave drops its 16 bytes at LDS base + 16 L), one whole 128-byte
// cache line per row and stage, two 64 KB stages.  The 16-byte chunk c of row r
// sits at chunk position c ^ ((r >> 1) & 7), which spreads the 16 rows that one
// pass of a ds_read_b128 touches over all 64 banks.  The loads are issued from
// inline asm so that their completion is awaited by explicit vmcnt counts; the
// compiler would otherwise wait for all of them at every barrier.
//
// One stage is four k sub-steps of 16 multiplies (bf16; 64 for fp32).  All LDS
// reads of a stage are issued, one after each multiply, by the end of sub-step 1,
// so the barrier that frees the stage's buffer sits early in sub-step 2, and the
// 16 loads of stage s+2 go out one every other multiply over the rest of the stage:
// a wave issues in order, and a burst of loads backs up the memory pipeline and
// holds up the multiplies queued behind it.  sched_barrier keeps the compiler from
// re-clustering what is interleaved here by hand.
// ---------------------------------------------------------------------------
namespace pipe {

constexpr int TM = 256, TN = 256;        // tile rows (x_i) and columns (x_j)
constexpr int LINE = 128;                // bytes of k per row and stage
constexpr int STAGE = (TM + TN) * LINE;  // 64 KB
constexpr int NSTAGE = 2;
constexpr int LDS_BYTES = NSTAGE * STAGE;
constexpr int NLOAD = STAGE / (THREADS * CHUNK);   // 16 loads per lane and stage

__device__ __forceinline__ int swizzle(int row) { return (row >> 1) & 7; }

__device__ __forceinline__ void load_to_lds(const void *gptr, unsigned lds_addr)
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
// 4 bytes per lane: lane L's word lands at LDS address lds_addr + 4 L
__device__ __forceinline__ void load_dword_to_lds(const void *gptr, unsigned lds_addr)
{
    unsigned saved;
    asm volatile("s_mov_b32 %0, m0\n\t"
                 "s_mov_b32 m0, %2\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dword %1, off\n\t"
                 "s_mov_b32 m0, %0"
                 : "=&s"(saved)
                 : "v"(gptr), "s"(lds_addr)
                 : "memory");
}
template <int N> __device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void pin_schedule() { __builtin_amdgcn_sched_barrier(0); }

// Tile row (0..255 = x_i rows, 256..511 = x_j rows) and 16-byte chunk of the row's
// line that lane `lane` of wave `wave` fetches with its u-th load of a stage.
// Waves 0 and 1 fetch the x_i rows, waves 2 and 3 the x_j rows.
__device__ __forceinline__ void load_slot(int wave, int u, int lane, int *tile_row, int *chunk)
{
    const int row = (wave * NLOAD + u) * 8 + (lane >> 3);
    *tile_row = row;
    *chunk = (lane & 7) ^ swizzle(row);
}

struct Frags { uint4 v[8]; };   // v[0..3]: x_i fragments (32 rows each), v[4..7]: x_j fragments

// The multiplies of one k sub-step; hook(i) runs right after the i-th of the first 16.
template <typename T, typename Hook>
__device__ __forceinline__ void multiply(const Frags &f, f32x16 (&acc)[4][4], Hook hook)
{
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, f.v[a]), __builtin_bit_cast(bf16x8, f.v[4 + b]), acc[a][b], 0, 0, 0);
                pin_schedule();
                hook(a * 4 + b);
                pin_schedule();
            }
    } else {
        // four 32x32x2 products per fragment pair; lanes<32 carry k = e, lanes>=32 carry k = 4+e,
        // for both operands alike, so every k of the group is used exactly once
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const f32x4 va = __builtin_bit_cast(f32x4, f.v[a]);
                    const f32x4 vb = __builtin_bit_cast(f32x4, f.v[4 + b]);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], vb[e], acc[a][b], 0, 0, 0);
                    if (e == 0) {
                        pin_schedule();
                        hook(a * 4 + b);
                        pin_schedule();
                    }
                }
    }
}

template <typename T>
struct Pipe {
    unsigned char *lds;
    unsigned wave_dst;            // LDS address of this wave's first load of a stage
    int aoff, boff, sw16, hi16;   // this lane's fragment rows, its swizzle and k half, in bytes
    const unsigned char *gp[NLOAD];   // this lane's chunk of the next stage to load, per load slot

    __device__ __forceinline__ void init(unsigned char *lds_)
    {
        lds = lds_;
        const int tid = threadIdx.x, lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int wr = wave >> 1, wc = wave & 1;
        const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;
        wave_dst = lds_base + wave * (NLOAD * 1024);
        aoff = (wr * 128 + (lane & 31)) * LINE;
        boff = (TM + wc * 128 + (lane & 31)) * LINE;
        sw16 = swizzle(lane & 31) << 4;     // fragment rows differ from lane & 31 by multiples of 32
        hi16 = (lane >> 5) << 4;            // lanes 0-31 take the first 16 bytes of a 32-byte k group
    }
    __device__ __forceinline__ void load1(int buf, int u)
    {
        load_to_lds(gp[u], wave_dst + buf * STAGE + u * 1024);
        gp[u] += LINE;
    }
    // fragment i (0..3 x_i, 4..7 x_j) of k sub-step kk of the stage in buffer buf
    __device__ __forceinline__ void read1(Frags &f, int buf, int kk, int i)
    {
        const unsigned char *base = lds + buf * STAGE;
        const int pos = (kk * 32 + hi16) ^ sw16;
        if (i < 4) f.v[i] = *reinterpret_cast<const uint4 *>(base + aoff + pos + i * 32 * LINE);
        else f.v[i] = *reinterpret_cast<const uint4 *>(base + boff + pos + (i - 4) * 32 * LINE);
    }
    // Start the loads of a tile's first two stages (gp set, nstage >= 1).
    __device__ __forceinline__ void start(int nstage)
    {
#pragma unroll
        for (int u = 0; u < NLOAD; ++u) load1(0, u);
        if (nstage > 1) {
#pragma unroll
            for (int u = 0; u < NLOAD; ++u) load1(1, u);
        }
    }
    // The whole k loop of a tile whose start() has been called; acc = sum over all of k.
    // Ends with a barrier: the ring is free in every wave.
    __device__ __forceinline__ void run(int nstage, f32x16 (&acc)[4][4])
    {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
        if (nstage > 1) wait_loads<NLOAD>();
        else wait_loads<0>();
        __builtin_amdgcn_s_barrier();
        Frags f0, f1, f2, f3;     // k sub-steps 0..3 of the current stage
#pragma unroll
        for (int i = 0; i < 8; ++i) read1(f0, 0, 0, i);
        auto nothing = [](int) {};
        int buf = 0;
        // MORE: another stage follows.  REFILL: stage s+2 exists and takes this stage's buffer.
        auto stage = [&](auto more_tag, auto refill_tag) {
            constexpr bool MORE = decltype(more_tag)::value, REFILL = decltype(refill_tag)::value;
            multiply<T>(f0, acc, [&](int i) { if (i < 8) read1(f1, buf, 1, i); });
            multiply<T>(f1, acc, [&](int i) {
                if (i < 8) read1(f2, buf, 2, i);
                else read1(f3, buf, 3, i - 8);
            });
            if constexpr (MORE) {
                multiply<T>(f2, acc, [&](int i) {
                    if (i == 3) {
                        // my loads of stage s+1 have landed and my reads of stage s are complete;
                        // after the barrier that holds for every wave
                        wait_loads<0>();
                        wait_lds();
                        __builtin_amdgcn_s_barrier();
                    }
                    if constexpr (REFILL)
                        if (i >= 4 && (i & 1) == 0) load1(buf, (i - 4) >> 1);     // loads 0..5
                });
                multiply<T>(f3, acc, [&](int i) {
                    if (i < 8) read1(f0, buf ^ 1, 0, i);
                    if constexpr (REFILL)
                        if (i < 10) load1(buf, 6 + i);                            // loads 6..15
                });
            } else {
                multiply<T>(f2, acc, nothing);
                multiply<T>(f3, acc, nothing);
            }
            buf ^= 1;
        };
        int s = 0;
        for (; s + 2 < nstage; ++s) stage(std::true_type{}, std::true_type{});
        if (s + 1 < nstage) stage(std::true_type{}, std::false_type{});
        stage(std::false_type{}, std::false_type{});
        wait_lds();
        __builtin_amdgcn_s_barrier();
    }
};

// One accumulator element, fetched from the accumulator register file at the point of use.
// The explicit read keeps the register allocator from moving a whole tile's 256 accumulators
// into ordinary registers at once, which leaves room for nothing else.
__device__ __forceinline__ float acc_read(float a)
{
    float v;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// The workgroups of a launch are dealt round-robin to the 8 XCDs, each with an L2 of its own.
// Tile number t of workgroup w: every XCD owns a contiguous run of the tile list, and the
// list walks the tile grid in bands of 8 tile rows, down the band first, so that the 32
// workgroups an XCD runs side by side share their feature rows in its L2.
__device__ __forceinline__ bool tile_of_workgroup(int w, int nwg, int tiles_m, int tiles_n, int *ti, int *tj)
{
    const int per = (nwg + 7) >> 3;
    const int t = (w & 7) * per + (w >> 3);
    if (t >= tiles_m * tiles_n) return false;
    constexpr int BAND = 8;
    const int band = t / (BAND * tiles_n);
    const int rows_in_band = min(BAND, tiles_m - band * BAND);
    const int r = t - band * BAND * tiles_n;
    *ti = band * BAND + r % rows_in_band;
    *tj = r / rows_in_band;
    return true;
}

} // namespace pipe

// Gram tile + Gaussian epilogue, fast path.  grid = tiles rounded up to a multiple of 8,
// dynamic LDS = pipe::LDS_BYTES.  Columns n .. ncols_pad-1 of the output are written as 0.
// EPI = EPI_RBF_MIRROR: S is symmetric, so only the tiles on and above the diagonal are computed (the same
// folded tile list as below, same grid) and each one above the diagonal also stores its transpose; needs
// ncols_pad <= 256 * ceil(n / 256), S 16-byte aligned and lds_out a multiple of 4.
// EPI = EPI_DISTANCE: nothing is stored; the sum of the tile's distances over its pairs i < j goes to
// one slot of pair_sums; call with exp_scale = 1, ncols_pad = n and a grid of
// ((tiles + 1) / 2) * (tiles + 1) workgroups rounded up to a multiple of 8, tiles = ceil(n / 256),
// which is also the number of slots.
// The body: workgroup `wg` of the `nwg` that share one matrix (a launch may hold several matrices).
template <typename T, int EPI>
__device__ __forceinline__ void
gram_rbf_fast_tile(const T *__restrict__ X, long long ldx, const int32_t *__restrict__ row_index, int n, int d,
                   const float *__restrict__ sq, float exp_scale, float *__restrict__ S, long long lds_out,
                   int ncols_pad, double *__restrict__ pair_sums, int wg, int nwg)
{
    using namespace pipe;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int tiles_m = (n + TM - 1) / TM, tiles_n = (ncols_pad + TN - 1) / TN;
    int ti, tj;
    size_t sum_slot = 0;
    if constexpr (EPI != EPI_RBF) {
        // Only tiles on or above the diagonal carry pairs (i < j).  Tile row r (tiles_m - r of them) and
        // tile row tiles_m - 1 - r (r + 1 of them) together fill one row of a (tiles_m + 1)-wide
        // rectangle with (tiles_m + 1) / 2 rows, which is dealt to the workgroups like any tile grid.
        int r, c;
        if (!tile_of_workgroup(wg, nwg, (tiles_m + 1) / 2, tiles_m + 1, &r, &c)) return;
        sum_slot = (size_t)r * (tiles_m + 1) + c;
        if (c < tiles_m - r) {
            ti = r;
            tj = r + c;
        } else {
            ti = tiles_m - 1 - r;
            tj = ti + (c - (tiles_m - r));
            if (ti == r) {
                // odd tile count: the middle tile row has no partner, its slots past the row's end stay empty
                if constexpr (EPI == EPI_DISTANCE)
                    if (tid == 0) pair_sums[sum_slot] = 0.0;
                return;
            }
        }
    } else {
        if (!tile_of_workgroup(wg, nwg, tiles_m, tiles_n, &ti, &tj)) return;
    }
    const int i0 = ti * TM, j0 = tj * TN;

    if constexpr (EPI != EPI_RBF) {
        // every tile of the list holds work
    } else if (j0 >= n) {
        // tile entirely in the zero padding of the output pitch
        for (int e = tid; e < TM * TN; e += THREADS) {
            const int i = i0 + e / TN, j = j0 + e % TN;
            if (i < n && j < ncols_pad) S[(size_t)i * lds_out + j] = 0.f;
        }
        return;
    }

    Pipe<T> p;
    p.init(lds);
#pragma unroll
    for (int u = 0; u < NLOAD; ++u) {
        int trow, chunk;
        load_slot(wave, u, lane, &trow, &chunk);
        const int gi = trow < TM ? min(i0 + trow, n - 1) : min(j0 + trow - TM, n - 1);
        const int row = row_index ? row_index[gi] : gi;
        p.gp[u] = reinterpret_cast<const unsigned char *>(X + (size_t)row * ldx) + chunk * CHUNK;
    }
    const int nstage = (int)(((long long)d * (int)sizeof(T)) / LINE);
    p.start(nstage);
    // what the epilogue needs from memory is fetched under the k loop
    const float my_sq_row = (i0 + tid < n) ? sq[i0 + tid] * exp_scale : 0.f;
    float sqj[4];
    int jj[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        jj[b] = j0 + wc * 128 + b * 32 + (lane & 31);
        sqj[b] = jj[b] < n ? sq[jj[b]] * exp_scale : 0.f;
    }
    f32x16 acc[4][4];
    p.run(nstage, acc);

    // epilogue: a lane holds column (lane & 31) of each 32-wide block b, rows
    // 32 a + 8 rq + 4 (lane >> 5) + e.  The row norms go through LDS (the ring is idle).
    float *sq_rows = reinterpret_cast<float *>(lds);
    sq_rows[tid] = my_sq_row;
    __syncthreads();
    const float scale2 = -2.f * exp_scale;
    const int r0 = i0 + wr * 128 + (lane >> 5) * 4;
    if constexpr (EPI == EPI_DISTANCE) {
        double total = 0.0;
        auto sum_up = [&](auto plain_tag) {
            constexpr bool PLAIN = decltype(plain_tag)::value;   // interior tile above the diagonal: every pair counts
            int i = r0;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int rl = wr * 128 + a * 32 + rq * 8 + (lane >> 5) * 4;
                    const float4 sqi4 = *reinterpret_cast<const float4 *>(sq_rows + rl);
                    const float sqi[4] = {sqi4.x, sqi4.y, sqi4.z, sqi4.w};
                    float part = 0.f;      // 16 distances at a time in fp32, then into the double
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            float dist = distance_value(acc_read(acc[a][b][rq * 4 + e]), sqi[e], sqj[b]);
                            if constexpr (!PLAIN) dist = (jj[b] > i && jj[b] < n) ? dist : 0.f;
                            part += dist;
                        }
                        i += (e == 3) ? 5 : 1;
                    }
                    total += (double)part;
                    asm volatile("" : "+v"(total));      // the sum is taken here, not saved up for the end
                    pin_schedule();
                }
            }
        };
        if (i0 + TM <= n && j0 + TN <= n && tj > ti) sum_up(std::true_type{});
        else sum_up(std::false_type{});
        tile_distance_sum(total, reinterpret_cast<double *>(lds + 2048), tid, &pair_sums[sum_slot]);
        return;
    }
    float *dst0 = S + (size_t)r0 * lds_out + (j0 + wc * 128 + (lane & 31));
    // one running row pointer per lane: rows advance +1 +1 +1 +5 through the accumulator layout
    const long long step1 = lds_out, step5 = 5 * lds_out;
    // EPI_RBF_MIRROR: a tile above the diagonal also writes its transpose, S(j,i) = S(i,j).  A lane's four
    // consecutive rows of one column are four consecutive floats of the mirrored row; stored straight
    // from the registers they leave as 16-byte pieces of 32 different lines per instruction (measured: the
    // 50 000 x 2048 build takes 9.1 ms that way against 5.6 ms).  An
    // interior tile therefore turns each 32-row band of a wave's sub-tile round in LDS (the ring is
    // idle; a wave has a region of its own, 128 mirrored rows of 32 floats at a pitch of 36) and stores
    // it as whole 128-byte lines, eight per instruction.  Edge tiles store element by element, checked.
    constexpr int TP = 36;
    float *mir[4];
    float *turn = nullptr, *mir_lines = nullptr;
    if constexpr (EPI == EPI_RBF_MIRROR) {
#pragma unroll
        for (int b = 0; b < 4; ++b) mir[b] = S + (size_t)min(jj[b], n - 1) * lds_out + r0;
        turn = reinterpret_cast<float *>(lds + 4096) + wave * (128 * TP);
        // lane -> mirrored row (lane >> 3) of a group of eight, floats 4 (lane & 7) .. + 3 of the band
        mir_lines = S + (size_t)min(j0 + wc * 128 + (lane >> 3), n - 1) * lds_out + (i0 + wr * 128 + (lane & 7) * 4);
    }
    const bool mirror = EPI == EPI_RBF_MIRROR && ti != tj;
    auto epilogue = [&](auto plain_tag) {
        constexpr bool PLAIN = decltype(plain_tag)::value;   // interior tile off the diagonal: no checks
        float *dst = dst0;
        int i = r0;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int rl = wr * 128 + a * 32 + rq * 8 + (lane >> 5) * 4;
                const float4 sqi4 = *reinterpret_cast<const float4 *>(sq_rows + rl);
                const float sqi[4] = {sqi4.x, sqi4.y, sqi4.z, sqi4.w};
                float col[4][4];        // [b][e]: what goes to the mirrored rows
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        float v = rbf_value(acc_read(acc[a][b][rq * 4 + e]), sqi[e], sqj[b], scale2);
                        if constexpr (PLAIN) {
                            __builtin_nontemporal_store(v, dst + b * 32);
                        } else {
                            if (i == jj[b]) v = 1.f;
                            if (i < n && jj[b] < ncols_pad) dst[b * 32] = jj[b] < n ? v : 0.f;
                        }
                        col[b][e] = v;
                    }
                    dst += (e == 3) ? step5 : step1;
                    i += (e == 3) ? 5 : 1;
                }
                if constexpr (EPI == EPI_RBF_MIRROR) {
                    if constexpr (PLAIN) {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            *reinterpret_cast<float4 *>(turn + (b * 32 + (lane & 31)) * TP + rq * 8 + (lane >> 5) * 4) =
                                make_float4(col[b][0], col[b][1], col[b][2], col[b][3]);
                    } else if (mirror) {
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            float *m = mir[b] + (a * 32 + rq * 8);
                            const int ib = i0 + rl;       // the four rows i of this group are the columns here
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (jj[b] < n && ib + e < n) m[e] = col[b][e];
                        }
                    }
                }
                pin_schedule();
            }
            if constexpr (EPI == EPI_RBF_MIRROR && PLAIN) {
                // the band is complete in this wave's region (LDS operations of one wave stay in order)
                float *out = mir_lines + a * 32;
#pragma unroll
                for (int g = 0; g < 16; ++g) {
                    const float4 line = *reinterpret_cast<const float4 *>(turn + (g * 8 + (lane >> 3)) * TP + (lane & 7) * 4);
                    __builtin_nontemporal_store(__builtin_bit_cast(f32x4, line), reinterpret_cast<f32x4 *>(out + (size_t)(g * 8) * lds_out));
                }
                pin_schedule();
            }
        }
    };
    if (i0 + TM <= n && j0 + TN <= n && ti != tj) epilogue(std::true_type{});
    else epilogue(std::false_type{});
}

template <typename T, int EPI = EPI_RBF>
__global__ void __launch_bounds__(THREADS, 1)
k_gram_rbf_fast(const T *__restrict__ X, long long ldx, const int32_t *__restrict__ row_index, int n, int d,
                const float *__restrict__ sq, float exp_scale, float *__restrict__ S, long long lds_out,
                int ncols_pad, double *__restrict__ pair_sums)
{
    gram_rbf_fast_tile<T, EPI>(X, ldx, row_index, n, d, sq, exp_scale, S, lds_out, ncols_pad, pair_sums,
                               (int)blockIdx.x, (int)gridDim.x);
}

// Several similarity matrices over the same feature matrix in one launch (the classes of a data set: a
// class of a few hundred samples is a handful of tiles, and one launch per class would leave the chip
// idle).  The jobs travel in the kernel arguments.  Job j owns workgroups wg_begin .. wg_begin + wg_count
// (both multiples of 8, so a job's workgroups meet the XCDs the way a launch of its own would) and, in
// the row-norm launch, workgroups row_wg_begin .. of four rows each.
constexpr int SIM_BATCH = 64;
struct SimJob {
    const int32_t *row_index;
    float *sq;
    float *S;
    long long lds_out;
    int n, ncols_pad;
    int wg_begin, wg_count;
    int row_wg_begin, pad_;
};
struct SimBatch {
    SimJob job[SIM_BATCH];
    int njobs;
};

template <typename T, int EPI>
__global__ void __launch_bounds__(THREADS, 1)
k_gram_rbf_fast_batch(const T *__restrict__ X, long long ldx, int d, float exp_scale, const SimBatch b)
{
    const int wg = (int)blockIdx.x;
    int j = 0;
    while (j + 1 < b.njobs && wg >= b.job[j + 1].wg_begin) ++j;
    const SimJob &q = b.job[j];
    gram_rbf_fast_tile<T, EPI>(X, ldx, q.row_index, q.n, d, q.sq, exp_scale, q.S, q.lds_out, q.ncols_pad, nullptr,
                               wg - q.wg_begin, q.wg_count);
}

template <typename T>
__global__ void __launch_bounds__(256)
k_row_norms_batch(const T *__restrict__ X, long long ldx, int d, const SimBatch b)
{
    const int wg = (int)blockIdx.x;
    int j = 0;
    while (j + 1 < b.njobs && wg >= b.job[j + 1].row_wg_begin) ++j;
    const SimJob &q = b.job[j];
    const int lane = threadIdx.x & 63;
    const int i = (wg - q.row_wg_begin) * 4 + (threadIdx.x >> 6);
    if (i >= q.n) return;
    const int r = q.row_index ? q.row_index[i] : i;
    const T *p = X + (size_t)r * ldx;
    double a = 0.0;
    for (int t = lane; t < d; t += 64) {
        const double v = (double)to_f32(p[t]);
        a += v * v;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);
    if (lane == 0) q.sq[i] = (float)a;
}

// Gram tile + Gaussian epilogue, general path (any alignment, any d).  grid = (column tiles, row tiles).
// EPI = EPI_DISTANCE: the tile's distance sum goes to pair_sums[blockIdx.y * gridDim.x + blockIdx.x]
// (exp_scale = 1, ncols_pad = n).
template <typename T, int EPI = EPI_RBF>
__global__ void __launch_bounds__(THREADS, 2)
k_gram_rbf(const T *__restrict__ X, long long ldx, const int32_t *__restrict__ row_index, int n, int d,
           const float *__restrict__ sq, float exp_scale, float *__restrict__ S, long long lds_out,
           int ncols_pad, double *__restrict__ pair_sums)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BN;

    if constexpr (EPI == EPI_DISTANCE) {
        if (j0 + BN <= i0 + 1) {
            // no column of this tile lies right of the diagonal: its pairs are counted from the other side
            if (tid == 0) pair_sums[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = 0.0;
            return;
        }
    } else if (j0 >= n) {
        // tile entirely in the zero padding of the output pitch
        for (int e = tid; e < BM * BN; e += THREADS) {
            const int i = i0 + e / BN, j = j0 + e % BN;
            if (i < n && j < ncols_pad) S[(size_t)i * lds_out + j] = 0.f;
        }
        return;
    }

    f32x16 acc[4][2];
    {
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
        gram_mainloop<T>(X, ldx, d, vec_ok, arow, brow, lds, acc);
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
    if constexpr (EPI == EPI_DISTANCE) {
        double total = 0.0;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int j = j0 + wc * 64 + b * 32 + (lane & 31);
            const float sqj = j < n ? sq[j] : 0.f;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int rl = wr * 128 + a * 32 + rq * 8 + (lane >> 5) * 4;
                    const float4 sqi4 = *reinterpret_cast<const float4 *>(sq_rows + rl);
                    const float sqi[4] = {sqi4.x, sqi4.y, sqi4.z, sqi4.w};
                    float part = 0.f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float dist = distance_value(acc[a][b][rq * 4 + e], sqi[e], sqj);
                        part += (j > i0 + rl + e && j < n) ? dist : 0.f;
                    }
                    total += (double)part;
                }
            }
        }
        tile_distance_sum(total, reinterpret_cast<double *>(lds + 2048), tid,
                          &pair_sums[(size_t)blockIdx.y * gridDim.x + blockIdx.x]);
        return;
    }
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

// out[0] = sum of count doubles, in a fixed order: one workgroup, strided partial sums, then a tree.
__global__ void __launch_bounds__(1024)
k_sum_doubles(const double *__restrict__ v, long long count, double *__restrict__ out)
{
    __shared__ double part[1024];
    double a = 0.0;
    for (long long i = threadIdx.x; i < count; i += 1024) a += v[i];
    part[threadIdx.x] = a;
    __syncthreads();
    for (int w = 512; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = part[0];
}

} // namespace sim
