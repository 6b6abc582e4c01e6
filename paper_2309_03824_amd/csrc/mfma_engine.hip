// bf16 MFMA engine for gfx950: LDS-tiled matrix products on v_mfma_f32_32x32x16_bf16 with fp32
// accumulation.  Two kernels:
//   gemm_kernel   one product, either operand stored k-contiguous or k-major (transposed while
//                 it is staged into LDS), optional split-K into fp32 partials;
//   chain_kernel  two products back to back through a rank-R intermediate that is produced into
//                 LDS and consumed from there (the low-rank pair: X.V^T -> H -> H.U^T, and its
//                 data-gradient mirror dY.U -> dH -> dH.V), so H never makes a round trip to HBM.
//
// Tiling: 256 threads = 4 wavefronts of 64 lanes in a 2 x 2 arrangement; each wavefront owns
// 32 x 32 MFMA tiles of the workgroup tile.  K advances in steps of 64 elements through two LDS
// buffers; global loads for step k+1 are issued before the MFMAs of step k and written to LDS
// after them (one barrier per step).  LDS rows are padded by 16 bytes so that the 16-byte operand
// reads of a wavefront spread over all banks.
//
// MFMA operand roles are swapped on purpose (the N-side fragment is passed first): the
// accumulator of a lane then holds, for ONE output row m, groups of 4 consecutive columns n,
// which turns the epilogue into 8-byte (bf16) / 16-byte (fp32) row-major stores.
#include "lrd_internal.hpp"

namespace lrd {
namespace {

constexpr int NTHREADS = 256;
constexpr int BK = 64;          // k elements per LDS stage
constexpr int LDK = BK + 8;     // padded LDS row length (elements)
constexpr int BN2 = 128;        // output columns per step of the chain's second product

// One operand as the kernels see it.  k-contiguous: element (row,k) = p[row*ld + k];
// k-major: element (row,k) = p[k*ld + row].  `vec` = widest load (in elements: 8,4,2,1) that base
// alignment, ld and the contiguous extent allow.
struct Src {
    const bf16_t* p;
    int64_t ld;
    int rows;
    int K;
    int vec;
};

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// 8 consecutive bf16 starting at p, of which the first `valid` exist; the rest read as zero.
__device__ __forceinline__ u32x4 load8(const bf16_t* p, int valid, int vec)
{
    u32x4 v = {0u, 0u, 0u, 0u};
    if (valid <= 0) return v;
    if (vec == 8) {
        v = *reinterpret_cast<const u32x4*>(p);
    } else if (vec == 4) {
        u32x2 a = *reinterpret_cast<const u32x2*>(p);
        v.x = a.x; v.y = a.y;
        if (valid > 4) {
            u32x2 b = *reinterpret_cast<const u32x2*>(p + 4);
            v.z = b.x; v.w = b.y;
        }
    } else if (vec == 2) {
        const uint32_t* s = reinterpret_cast<const uint32_t*>(p);
        v.x = s[0];
        if (valid > 2) v.y = s[1];
        if (valid > 4) v.z = s[2];
        if (valid > 6) v.w = s[3];
    } else {
        const uint16_t* s = reinterpret_cast<const uint16_t*>(p);
        uint32_t e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = (valid > q) ? (uint32_t)s[q] : 0u;
        v.x = e[0] | (e[1] << 16); v.y = e[2] | (e[3] << 16);
        v.z = e[4] | (e[5] << 16); v.w = e[6] | (e[7] << 16);
    }
    return v;
}

// ---- k-contiguous operand: ROWS x BK tile, one 16-byte chunk = 8 k of one row -----------------
template <int ROWS>
struct KcStage {
    static constexpr int N = ROWS * 8 / NTHREADS;
    u32x4 v[N];
};

template <int ROWS>
__device__ __forceinline__ void kc_load(KcStage<ROWS>& s, const Src& src, int row0, int k0, int tid)
{
#pragma unroll
    for (int i = 0; i < KcStage<ROWS>::N; ++i) {
        int c = tid + i * NTHREADS;
        int row = row0 + (c >> 3), k = k0 + (c & 7) * 8;
        int valid = (row < src.rows) ? min(8, src.K - k) : 0;
        s.v[i] = load8(src.p + (int64_t)row * src.ld + k, valid, src.vec);
    }
}

template <int ROWS>
__device__ __forceinline__ void kc_store(const KcStage<ROWS>& s, bf16_t* lds, int tid)
{
#pragma unroll
    for (int i = 0; i < KcStage<ROWS>::N; ++i) {
        int c = tid + i * NTHREADS;
        *reinterpret_cast<u32x4*>(lds + (c >> 3) * LDK + (c & 7) * 8) = s.v[i];
    }
}

// ---- k-major operand: BK x COLS tile read in units of 8 k x 8 columns, transposed in registers
template <int COLS>
struct KmStage {
    static constexpr int N = (COLS + NTHREADS - 1) / NTHREADS;
    u32x4 v[N][8];
};

template <int COLS>
__device__ __forceinline__ void km_load(KmStage<COLS>& s, const Src& src, int col0, int k0, int tid)
{
#pragma unroll
    for (int i = 0; i < KmStage<COLS>::N; ++i) {
        int u = tid + i * NTHREADS;
        if (COLS < NTHREADS && u >= COLS) continue;
        int kb = u & 7, nb = u >> 3;
        int col = col0 + nb * 8;
        int validc = min(8, src.rows - col);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int k = k0 + kb * 8 + e;
            s.v[i][e] = load8(src.p + (int64_t)k * src.ld + col, (k < src.K) ? validc : 0, src.vec);
        }
    }
}

template <int COLS>
__device__ __forceinline__ void km_store(const KmStage<COLS>& s, bf16_t* lds, int tid)
{
#pragma unroll
    for (int i = 0; i < KmStage<COLS>::N; ++i) {
        int u = tid + i * NTHREADS;
        if (COLS < NTHREADS && u >= COLS) continue;
        int kb = u & 7, nb = u >> 3;
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            u32x4 o;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t a = s.v[i][2 * q][n >> 1], b = s.v[i][2 * q + 1][n >> 1];
                o[q] = (n & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
            }
            *reinterpret_cast<u32x4*>(lds + (nb * 8 + n) * LDK + kb * 8) = o;
        }
    }
}

template <int ROWS, bool KM>
struct Stage;
template <int ROWS>
struct Stage<ROWS, false> {
    KcStage<ROWS> s;
    __device__ __forceinline__ void load(const Src& src, int row0, int k0, int tid) { kc_load<ROWS>(s, src, row0, k0, tid); }
    __device__ __forceinline__ void store(bf16_t* lds, int tid) const { kc_store<ROWS>(s, lds, tid); }
};
template <int ROWS>
struct Stage<ROWS, true> {
    KmStage<ROWS> s;
    __device__ __forceinline__ void load(const Src& src, int row0, int k0, int tid) { km_load<ROWS>(s, src, row0, k0, tid); }
    __device__ __forceinline__ void store(bf16_t* lds, int tid) const { km_store<ROWS>(s, lds, tid); }
};

// ---- one BK step of MFMAs on LDS tiles ---------------------------------------------------------
// a_lds: rows = output rows m (stride lda elements), b_lds: rows = output columns n (stride LDK).
template <int TM, int TN>
__device__ __forceinline__ void mma_step(f32x16 (&acc)[TM][TN], const bf16_t* a_lds, int lda, const bf16_t* b_lds,
                                         int lane)
{
    const int r = lane & 31, kh = (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(a_lds + (i * 32 + r) * lda + kk * 16 + kh);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(b_lds + (j * 32 + r) * LDK + kk * 16 + kh);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(b[j], a[i], acc[i][j]);
    }
}

template <int TM, int TN>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[TM][TN])
{
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
}

// Store 4 consecutive columns of one row.  cvec >= 4: the row start and n are 4-aligned and the
// whole group is inside N, so one vector store does it; otherwise element by element.
__device__ __forceinline__ void store4(bf16_t* row, int n, int N, f32x4 v, int cvec)
{
    if (cvec >= 4 && n + 3 < N) {
        u32x2 pk = {pack_bf16(v.x, v.y), pack_bf16(v.z, v.w)};
        *reinterpret_cast<u32x2*>(row + n) = pk;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n + e < N) row[n + e] = (bf16_t)v[e];
    }
}

__device__ __forceinline__ void store4(float* row, int n, int N, f32x4 v, int cvec)
{
    if (cvec >= 4 && n + 3 < N) {
        *reinterpret_cast<f32x4*>(row + n) = v;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n + e < N) row[n + e] = v[e];
    }
}

// Accumulators of one wavefront -> row-major C.  (m_base, n_base) = origin of the wavefront tile.
template <int TM, int TN, class OutT>
__device__ __forceinline__ void store_tiles(const f32x16 (&acc)[TM][TN], OutT* C, int64_t ldc, int m_base, int n_base,
                                            int M, int N, const float* bias, int cvec, int lane)
{
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int m = m_base + i * 32 + r;
        if (m >= M) continue;
        OutT* row = C + (int64_t)m * ldc;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int n = n_base + j * 32 + 8 * g + 4 * h;
                if (n >= N) continue;
                f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                if (bias) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) v[e] += bias[n + e];
                }
                store4(row, n, N, v, cvec);
            }
    }
}

// ================================================================================================
// Single product
// ================================================================================================
template <int BM, int BN, bool A_KM, bool B_KM, class OutT>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(Src A, Src B, OutT* C, int64_t ldc, const float* bias,
                                                        float* partial, int M, int N, int k_per_split, int cvec)
{
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(smem);
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int STAGE = (BM + BN) * LDK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int kbeg = blockIdx.z * k_per_split;
    const int kend = min(A.K, kbeg + k_per_split);
    A.K = kend;
    B.K = kend;

    f32x16 acc[TM][TN];
    zero_acc<TM, TN>(acc);

    Stage<BM, A_KM> sa;
    Stage<BN, B_KM> sb;
    const int nk = (kend - kbeg + BK - 1) / BK;
    if (nk > 0) {
        sa.load(A, m0, kbeg, tid);
        sb.load(B, n0, kbeg, tid);
        sa.store(lds, tid);
        sb.store(lds + BM * LDK, tid);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        bf16_t* cur = lds + (kt & 1) * STAGE;
        bf16_t* nxt = lds + ((kt + 1) & 1) * STAGE;
        const bool more = kt + 1 < nk;
        if (more) {
            sa.load(A, m0, kbeg + (kt + 1) * BK, tid);
            sb.load(B, n0, kbeg + (kt + 1) * BK, tid);
        }
        mma_step<TM, TN>(acc, cur + wm * (BM / 2) * LDK, LDK, cur + BM * LDK + wn * (BN / 2) * LDK, lane);
        if (more) {
            sa.store(nxt, tid);
            sb.store(nxt + BM * LDK, tid);
        }
        __syncthreads();
    }

    if (partial) {
        float* P = partial + (int64_t)blockIdx.z * M * N;
        store_tiles<TM, TN, float>(acc, P, N, m0 + wm * (BM / 2), n0 + wn * (BN / 2), M, N, nullptr, (N % 4 == 0) ? 4 : 1,
                                   lane);
    } else {
        store_tiles<TM, TN, OutT>(acc, C, ldc, m0 + wm * (BM / 2), n0 + wn * (BN / 2), M, N, bias, cvec, lane);
    }
}

// ================================================================================================
// Two products through an on-chip rank-R intermediate
// ================================================================================================
template <int BM, int RP>
constexpr int chain_lds_bytes()
{
    constexpr int s1 = 2 * (BM + RP) * LDK;
    constexpr int s2 = BM * (RP + 8) + 2 * BN2 * LDK;
    return (s1 > s2 ? s1 : s2) * 2;
}

template <int BM, int RP, bool B1_KM, bool B2_KM>
__global__ __launch_bounds__(NTHREADS) void chain_kernel(Src A, Src B1, Src B2, bf16_t* C, int64_t ldc, bf16_t* mid,
                                                         int64_t ldmid, const float* bias, int M, int R, int N2,
                                                         int cvec, int midvec)
{
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(smem);
    constexpr int TM = BM / 64;         // 32-row tiles per wavefront (both products)
    constexpr int TN1 = RP / 64;        // first product: wavefront owns RP/2 columns of H
    constexpr int TN2 = BN2 / 64;       // second product: wavefront owns 64 of the 128 columns
    constexpr int STAGE1 = (BM + RP) * LDK;
    constexpr int LDH = RP + 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * BM;

    // ---- product 1: H[BM x RP] = A[BM x K1] . B1^T --------------------------------------------
    {
        f32x16 acc[TM][TN1];
        zero_acc<TM, TN1>(acc);
        Stage<BM, false> sa;
        Stage<RP, B1_KM> sb;
        const int nk = (A.K + BK - 1) / BK;
        sa.load(A, m0, 0, tid);
        sb.load(B1, 0, 0, tid);
        sa.store(lds, tid);
        sb.store(lds + BM * LDK, tid);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            bf16_t* cur = lds + (kt & 1) * STAGE1;
            bf16_t* nxt = lds + ((kt + 1) & 1) * STAGE1;
            const bool more = kt + 1 < nk;
            if (more) {
                sa.load(A, m0, (kt + 1) * BK, tid);
                sb.load(B1, 0, (kt + 1) * BK, tid);
            }
            mma_step<TM, TN1>(acc, cur + wm * (BM / 2) * LDK, LDK, cur + BM * LDK + wn * (RP / 2) * LDK, lane);
            if (more) {
                sa.store(nxt, tid);
                sb.store(nxt + BM * LDK, tid);
            }
            __syncthreads();
        }
        // H -> LDS (bf16, row-major [BM][LDH]) and, if asked for, to global memory.
        const int r = lane & 31, h = lane >> 5;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int ml = wm * (BM / 2) + i * 32 + r;
            int m = m0 + ml;
#pragma unroll
            for (int j = 0; j < TN1; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    int c = wn * (RP / 2) + j * 32 + 8 * g + 4 * h;
                    f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    u32x2 pk = {pack_bf16(v.x, v.y), pack_bf16(v.z, v.w)};
                    *reinterpret_cast<u32x2*>(lds + ml * LDH + c) = pk;
                    if (mid && m < M && c < R) store4(mid + (int64_t)m * ldmid, c, R, v, midvec);
                }
        }
    }
    __syncthreads();

    // ---- product 2: C[BM x N2] = H . B2^T, 128 output columns at a time -------------------------
    {
        bf16_t* hs = lds;
        bf16_t* bs = lds + BM * LDH;
        constexpr int KT2 = RP / BK;
        const int nchunks = (N2 + BN2 - 1) / BN2;
        const int iters = nchunks * KT2;
        f32x16 acc[TM][TN2];
        zero_acc<TM, TN2>(acc);
        Stage<BN2, B2_KM> sb;
        sb.load(B2, 0, 0, tid);
        sb.store(bs, tid);
        __syncthreads();
        for (int it = 0; it < iters; ++it) {
            const int nc = it / KT2, kc = it - nc * KT2;
            bf16_t* cur = bs + (it & 1) * (BN2 * LDK);
            bf16_t* nxt = bs + ((it + 1) & 1) * (BN2 * LDK);
            const bool more = it + 1 < iters;
            if (more) {
                int nit = it + 1;
                int nnc = nit / KT2, nkc = nit - nnc * KT2;
                sb.load(B2, nnc * BN2, nkc * BK, tid);
            }
            mma_step<TM, TN2>(acc, hs + wm * (BM / 2) * LDH + kc * BK, LDH, cur + wn * (BN2 / 2) * LDK, lane);
            if (kc == KT2 - 1) {
                store_tiles<TM, TN2, bf16_t>(acc, C, ldc, m0 + wm * (BM / 2), nc * BN2 + wn * (BN2 / 2), M, N2, bias, cvec,
                                             lane);
                zero_acc<TM, TN2>(acc);
            }
            if (more) sb.store(nxt, tid);
            __syncthreads();
        }
    }
}

// ================================================================================================
// Host side
// ================================================================================================
inline int pow2_vec(uintptr_t base, int64_t ld, int64_t extent, int esz)
{
    int v = 8;
    while (v > 1 && ((base % (uintptr_t)(v * esz)) != 0 || ld % v != 0 || extent % v != 0)) v >>= 1;
    return v;
}

// Operand of a MatOp as a Src, or fails if neither stride is 1.
bool make_src(const void* p, int64_t s_row, int64_t s_k, int64_t rows, int64_t K, Src& out, bool& km)
{
    out.p = (const bf16_t*)p;
    out.rows = (int)rows;
    out.K = (int)K;
    if (s_k == 1) {
        km = false;
        out.ld = s_row;
        out.vec = pow2_vec((uintptr_t)p, s_row, K, 2);
        return true;
    }
    if (s_row == 1) {
        km = true;
        out.ld = s_k;
        out.vec = pow2_vec((uintptr_t)p, s_k, rows, 2);
        return true;
    }
    return false;
}

template <class K>
hipError_t allow_lds(K kernel, int bytes)
{
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

template <int BM, int BN, bool A_KM, bool B_KM, class OutT>
hipError_t launch_gemm(const MatOp& op, const Src& A, const Src& B, hipStream_t st)
{
    constexpr int lds_bytes = 2 * (BM + BN) * LDK * 2;
    auto kern = gemm_kernel<BM, BN, A_KM, B_KM, OutT>;
    static bool lds_allowed = false;   // per instantiation; setting it twice is harmless
    hipError_t e = hipSuccess;
    if (!lds_allowed) {
        e = allow_lds(kern, lds_bytes);
        if (e != hipSuccess) return e;
        lds_allowed = true;
    }
    int splits = (op.splits > 1 && op.partial) ? op.splits : 1;
    int kps = (int)(ceil_div(ceil_div(op.K, splits), BK) * BK);
    splits = (int)ceil_div(op.K, kps);
    float* partial = splits > 1 ? op.partial : nullptr;
    int cvec = pow2_vec((uintptr_t)op.C, op.ldc, op.N, (int)sizeof(OutT));
    dim3 grid((unsigned)ceil_div(op.M, BM), (unsigned)ceil_div(op.N, BN), (unsigned)splits);
    hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds_bytes, st, A, B, (OutT*)op.C, op.ldc, op.bias, partial,
                       (int)op.M, (int)op.N, kps, cvec);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (splits > 1) return reduce_partials(op.partial, op.C, false, op.ldc, op.M, op.N, splits, st, op.sgd);
    return hipSuccess;
}

template <int BM, int BN, class OutT>
hipError_t gemm_by_layout(const MatOp& op, const Src& A, bool akm, const Src& B, bool bkm, hipStream_t st)
{
    if (!akm && !bkm) return launch_gemm<BM, BN, false, false, OutT>(op, A, B, st);
    if (!akm && bkm) return launch_gemm<BM, BN, false, true, OutT>(op, A, B, st);
    if (akm && bkm) return launch_gemm<BM, BN, true, true, OutT>(op, A, B, st);
    return launch_gemm<BM, BN, true, false, OutT>(op, A, B, st);
}

}  // namespace

bool mfma_matop_supported(const MatOp& op)
{
    if (!op.in_bf16 || op.gather != GATHER_NONE) return false;
    if (op.M < 1 || op.N < 1 || op.K < 1) return false;
    if (op.M >= (int64_t(1) << 31) || op.N >= (int64_t(1) << 31) || op.K >= (int64_t(1) << 31)) return false;
    if (op.a_sk != 1 && op.a_sm != 1) return false;
    if (op.b_sk != 1 && op.b_sn != 1) return false;
    if (op.splits > 1 && !op.out_f32) return false;
    if (ceil_div(op.N, 64) > 65535) return false;
    return true;
}

hipError_t mfma_matop(const MatOp& op, hipStream_t st)
{
    note_kernel("gemm_kernel (any-alignment MFMA)");
    Src A, B;
    bool akm, bkm;
    if (!make_src(op.A, op.a_sm, op.a_sk, op.M, op.K, A, akm)) return hipErrorInvalidValue;
    if (!make_src(op.B, op.b_sn, op.b_sk, op.N, op.K, B, bkm)) return hipErrorInvalidValue;
    // Narrow outputs (a rank, a small channel count) take the 64-wide tile.
    const bool narrow = op.N <= 64 || (op.N > 128 && op.N <= 192);
    if (op.out_f32) {
        if (narrow) return gemm_by_layout<128, 64, float>(op, A, akm, B, bkm, st);
        return gemm_by_layout<128, 128, float>(op, A, akm, B, bkm, st);
    }
    if (narrow) return gemm_by_layout<128, 64, bf16_t>(op, A, akm, B, bkm, st);
    return gemm_by_layout<128, 128, bf16_t>(op, A, akm, B, bkm, st);
}

// ------------------------------------------------------------------------------------ chain
bool mfma_chain_supported(const ChainOp& op)
{
    if (op.R < 1 || op.R > 256) return false;
    if (op.M < 1 || op.K1 < 1 || op.N2 < 1) return false;
    if (op.M >= (int64_t(1) << 31) || op.K1 >= (int64_t(1) << 31) || op.N2 >= (int64_t(1) << 31)) return false;
    if (op.b1_sk != 1 && op.b1_sn != 1) return false;
    if (op.b2_sk != 1 && op.b2_sn != 1) return false;
    return true;
}

namespace {

template <int BM, int RP, bool B1_KM, bool B2_KM>
hipError_t launch_chain(const ChainOp& op, const Src& A, const Src& B1, const Src& B2, hipStream_t st)
{
    constexpr int lds_bytes = chain_lds_bytes<BM, RP>();
    auto kern = chain_kernel<BM, RP, B1_KM, B2_KM>;
    static bool lds_allowed = false;
    hipError_t e = hipSuccess;
    if (!lds_allowed) {
        e = allow_lds(kern, lds_bytes);
        if (e != hipSuccess) return e;
        lds_allowed = true;
    }
    int cvec = pow2_vec((uintptr_t)op.C, op.ldc, op.N2, 2);
    int midvec = op.mid_save ? pow2_vec((uintptr_t)op.mid_save, op.ldmid, op.R, 2) : 1;
    dim3 grid((unsigned)ceil_div(op.M, BM));
    hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds_bytes, st, A, B1, B2, (bf16_t*)op.C, op.ldc,
                       (bf16_t*)op.mid_save, op.ldmid, op.bias, (int)op.M, (int)op.R, (int)op.N2, cvec, midvec);
    return hipGetLastError();
}

template <int BM, int RP>
hipError_t chain_by_layout(const ChainOp& op, const Src& A, const Src& B1, bool b1km, const Src& B2, bool b2km,
                           hipStream_t st)
{
    if (!b1km && !b2km) return launch_chain<BM, RP, false, false>(op, A, B1, B2, st);
    if (b1km && b2km) return launch_chain<BM, RP, true, true>(op, A, B1, B2, st);
    if (!b1km && b2km) return launch_chain<BM, RP, false, true>(op, A, B1, B2, st);
    return launch_chain<BM, RP, true, false>(op, A, B1, B2, st);
}

template <int BM>
hipError_t chain_by_rank(const ChainOp& op, const Src& A, const Src& B1, bool b1km, const Src& B2, bool b2km,
                         hipStream_t st)
{
    if (op.R <= 64) return chain_by_layout<BM, 64>(op, A, B1, b1km, B2, b2km, st);
    if (op.R <= 128) return chain_by_layout<BM, 128>(op, A, B1, b1km, B2, b2km, st);
    if (op.R <= 192) return chain_by_layout<BM, 192>(op, A, B1, b1km, B2, b2km, st);
    return chain_by_layout<BM, 256>(op, A, B1, b1km, B2, b2km, st);
}

}  // namespace

hipError_t mfma_chain(const ChainOp& op, hipStream_t st)
{
    Src A, B1, B2;
    bool akm, b1km, b2km;
    if (!make_src(op.A, op.lda, 1, op.M, op.K1, A, akm)) return hipErrorInvalidValue;
    if (!make_src(op.B1, op.b1_sn, op.b1_sk, op.R, op.K1, B1, b1km)) return hipErrorInvalidValue;
    if (!make_src(op.B2, op.b2_sn, op.b2_sk, op.N2, op.R, B2, b2km)) return hipErrorInvalidValue;
    // 64-token tiles while that is what it takes to give every compute unit a workgroup.
    if (op.M <= 256 * 64) return chain_by_rank<64>(op, A, B1, b1km, B2, b2km, st);
    return chain_by_rank<128>(op, A, B1, b1km, B2, b2km, st);
}

}  // namespace lrd
