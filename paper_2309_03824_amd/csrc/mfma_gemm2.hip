// bf16 MFMA product kernel for 16-byte-aligned operands (the common case: every leading dimension
// a multiple of 8 elements).  One kernel template covers the three operand layouts of a layer:
//   forward / unfused pair      C = A . B^T          A [M x K], B [N x K]   (both k-contiguous)
//   data gradient               C = A . B            A [M x K], B [K x N]   (B k-major)
//   weight gradient (fp32 out)  C = A^T . B          A [K x M], B [K x N]   (both k-major), split-K
//
// Main loop: straight-line code, no data-dependent branches.  Every thread owns fixed 16-byte
// chunks of the operand tiles.  Plain operands are read with buffer loads whose range check returns
// zeros outside the operand (rows or columns that do not exist get an offset no descriptor admits);
// convolution gathers clamp the ADDRESS (so the load is always legal) and zero the VALUE when it is
// written to LDS.  Either way the loads have no consumers until the LDS hand-off and stay in flight
// across DEPTH K-steps; long reductions run a branch-free steady-state loop, the last steps a drain
// loop.  K-major operands are copied to LDS as they lie in memory and transposed by the LDS read
// (ds_read_b64_tr_b16) when the MFMA fragments are fetched, so no layout costs a VALU instruction.
// bf16 results leave through LDS so that each lane stores 16 contiguous bytes of an output row.
//
// Convolutions are the same kernel with gather tiles in place of the plain ones (implicit GEMM:
// forward, data gradient, weight gradient).  The data gradient of a strided convolution runs as one
// product per parity class of the input pixel (class = blockIdx.z), each over the taps that reach
// its pixels, and writes its rows through a row map.
#include <algorithm>
#include <cstdio>
#include <string>

#include "lrd_internal.hpp"

namespace lrd {
namespace {

constexpr int BK = 64;
constexpr int LDK = BK + 8;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

struct Operand {
    const bf16_t* p;
    int64_t ld;   // elements between rows of the stored matrix
    int rows;     // extent along the tile's row index (M for A, N for B)
};

// A batch of products of one shape in one launch (element strides between consecutive products).
struct BatchArgs {
    int batch = 1, nsplit = 1;
    int64_t a_bs = 0, b_bs = 0, c_bs = 0, aux_bs = 0, bias_bs = 0;
};

// Plain (strided) operands are read with buffer loads: the descriptor's base is the tile's first
// element for this K-step (wave-uniform), each chunk keeps one 32-bit byte offset, and the range
// check of the descriptor returns zeros for anything past the operand's last element.  A chunk
// whose row (or column group) does not exist gets an offset no descriptor admits, so static
// validity costs nothing per step; only the tail of K inside a row needs a mask, and only in the
// last step (store<true>).
constexpr uint32_t BUF_FLAGS = 0x00020000u;      // raw buffer, 32-bit data format
constexpr uint32_t BUF_OOB = 0xFFFFFFF0u;        // >= every num_records used here
constexpr int64_t BUF_MAX_LD = int64_t(1) << 22; // keeps (256 rows x ld + K) x 2 bytes below BUF_OOB

// Wave-uniform values the compiler cannot always prove uniform; a descriptor built from them stays
// in scalar registers instead of being looped over per distinct lane value.
__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uni64(int64_t v)
{
    uint64_t u = (uint64_t)v;
    return (int64_t)(((uint64_t)uni((uint32_t)(u >> 32)) << 32) | uni((uint32_t)u));
}
__device__ __forceinline__ const char* uni_ptr(const void* p)
{
    return reinterpret_cast<const char*>(uni64((int64_t)reinterpret_cast<uintptr_t>(p)));
}

__device__ __forceinline__ u32x4 buf_load16(const char* base, uint32_t span, uint32_t voff)
{
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, (int)span, (int)BUF_FLAGS);
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
}

// ---- k-contiguous tile: ROWS x BK, chunk c -> row c>>3, k-chunk c&7 ------------------------------
template <int ROWS, int NT, int DEPTH>
struct KcTile {
    static_assert(NT % 8 == 0, "every chunk of a thread has the same k offset");
    static constexpr int CH = (ROWS * 8 + NT - 1) / NT;
    static constexpr bool FULL = (ROWS * 8) % NT == 0;
    const char* base;     // first row of the tile, k = 0
    uint32_t span;        // bytes from base to the end of the tile's last existing row
    uint32_t voff[CH];
    int kc8;
    u32x4 st[DEPTH][CH];

    __device__ __forceinline__ void init(const Operand& o, int row0, int tid, const ConvShape&, int K, int)
    {
        base = uni_ptr(o.p + (int64_t)row0 * o.ld);
        const int rows_here = min(o.rows - row0, ROWS);
        span = uni((uint32_t)(((int64_t)(rows_here - 1) * o.ld + K) * 2));
        kc8 = (tid & 7) * 8;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int r = (tid + i * NT) >> 3;
            voff[i] = r < rows_here ? (uint32_t)((r * o.ld + kc8) * 2) : BUF_OOB;
        }
    }
    __device__ __forceinline__ void load(int d, int k0, int, int tid)
    {
        const uint32_t kb = uni((uint32_t)k0) * 2u;
        const char* b = base + kb;
        const uint32_t left = span - kb;      // k0 < K, so kb < span (a saturating form would leave the scalar unit)
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (FULL || tid + i * NT < ROWS * 8) st[d][i] = buf_load16(b, left, voff[i]);
    }
    template <bool TAIL>
    __device__ __forceinline__ void store(int d, bf16_t* lds, int k0, int kend, int tid) const
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        const bool inside = !TAIL || k0 + kc8 < kend;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            if (FULL || c < ROWS * 8)
                *reinterpret_cast<u32x4*>(lds + (c >> 3) * LDK + (c & 7) * 8) = inside ? st[d][i] : z;
        }
    }
};

// ---- k-major tile: BK x COLS kept in LDS as it is stored in memory ([k][column], columns
// contiguous); chunk c -> k = c / (COLS/8), column chunk c % (COLS/8).  The transposition the MFMA
// operand layout needs is done by the LDS read itself (ds_read_b64_tr_b16, see km_frag).
template <int COLS, int NT, int DEPTH>
struct KmTile {
    static constexpr int CPK = COLS / 8;                 // 16-byte chunks per k row
    static constexpr int LDM = COLS + 16;                // LDS row length: stride = 8 banks mod 32
    static constexpr int CH = (BK * CPK + NT - 1) / NT;
    static constexpr bool FULL = (BK * CPK) % NT == 0;
    const char* base;     // k = 0, first column of the tile
    int64_t ld;
    int K, cols_here;     // columns that exist from the tile's first one on
    uint32_t voff[CH];
    int krow[CH];
    u32x4 st[DEPTH][CH];

    __device__ __forceinline__ void init(const Operand& o, int col0, int tid, const ConvShape&, int Kdim, int)
    {
        ld = uni64(o.ld);
        K = (int)uni((uint32_t)Kdim);
        cols_here = (int)uni((uint32_t)(o.rows - col0));
        base = uni_ptr(o.p + col0);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            int col = (c % CPK) * 8;
            krow[i] = c / CPK;
            voff[i] = col < cols_here ? (uint32_t)((krow[i] * o.ld + col) * 2) : BUF_OOB;
        }
    }
    __device__ __forceinline__ void load(int d, int k0, int, int tid)
    {
        // bytes from this step's first k row to the last element of its last existing k row (at most
        // BK rows) in these columns; rows past K fall outside because ld >= cols_here
        const int ku = (int)uni((uint32_t)k0);
        const char* b = base + (int64_t)ku * ld * 2;
        const uint32_t left = (uint32_t)(min(K - ku, BK) - 1) * ((uint32_t)ld * 2u) + (uint32_t)cols_here * 2u;
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (FULL || tid + i * NT < BK * CPK) st[d][i] = buf_load16(b, left, voff[i]);
    }
    template <bool TAIL>
    __device__ __forceinline__ void store(int d, bf16_t* lds, int k0, int kend, int tid) const
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            if (FULL || c < BK * CPK)
                *reinterpret_cast<u32x4*>(lds + (c / CPK) * LDM + (c % CPK) * 8) =
                    (!TAIL || k0 + krow[i] < kend) ? st[d][i] : z;
        }
    }
};

// ---- implicit-GEMM operands of a k x k convolution on NHWC data ---------------------------------
// Same LDS layouts as the plain tiles; the address of a 16-byte chunk comes from the tap geometry,
// out-of-image taps and tails are clamped to a legal address and zeroed when the chunk is written
// to LDS.  Channel counts are multiples of 8 on this path, so a chunk never straddles two taps.
// K-steps are loaded strictly in order (k0 = kbeg, kbeg + BK, ...), so the decomposition of k into
// (tap, channel) or (image, y, x) is kept as state and advanced by BK after every load: the only
// integer divisions are in init().

// floor(t / d) for 0 <= t * d < 65536 by multiplication with ceil(65536 / d): taps by the kernel size
// (d < 32, t <= d * d + 8) and, in the data gradient, pixel coordinates by the stride.
__device__ __forceinline__ int small_div(int t, int magic) { return (t * magic) >> 16; }

// A operand, k-contiguous.  FWD:   row = output pixel, k = (u, v, i), reads X[n, y*s+u-p, x*s+v-p, i].
//                           DGRAD: row = input pixel,  k = (u, v, o), reads dY[n, (a+p-u)/s, (b+p-v)/s, o].
template <int ROWS, int NT, int DEPTH, bool DGRAD>
struct ConvRowsTile {
    static_assert(NT % 8 == 0, "every chunk of a thread has the same k offset");
    static constexpr int CH = (ROWS * 8 + NT - 1) / NT;
    static constexpr bool FULL = (ROWS * 8) % NT == 0;
    const bf16_t* base;
    ConvShape cs;
    int img[CH], py[CH], px[CH];
    bool rowok[CH];
    int kc8, tap, c0;         // this thread's k of the next load, as (tap, channel); same for all its chunks
    int ch, q_tap, r_ch, magic, magic_s;
    int kdiv, u0, v0, ustep;  // tap index -> (u, v): u = u0 + ustep * (tap / kdiv), v = v0 + ustep * (tap % kdiv)
    bool ok[DEPTH][CH];
    u32x4 st[DEPTH][CH];

    __device__ __forceinline__ void init(const Operand& o, int row0, int tid, const ConvShape& shape, int, int kbeg)
    {
        base = o.p;
        cs = shape;
        ch = DGRAD ? cs.O : cs.I;            // channels of the tensor being gathered
        q_tap = BK / ch;
        r_ch = BK - q_tap * ch;
        const bool cls = DGRAD && cs.cls;
        const ClassTaps tu = class_taps(cs.cy, cs.pad, cs.stride, cs.k), tv = class_taps(cs.cx, cs.pad, cs.stride, cs.k);
        kdiv = cls ? tv.count : cs.k;
        u0 = cls ? tu.first : 0;
        v0 = cls ? tv.first : 0;
        ustep = cls ? cs.stride : 1;
        magic = (65536 + kdiv - 1) / kdiv;
        magic_s = (65536 + cs.stride - 1) / cs.stride;
        kc8 = (tid & 7) * 8;
        tap = (kbeg + kc8) / ch;
        c0 = (kbeg + kc8) - tap * ch;
        // rows: output pixels, input pixels, or the input pixels of one parity class
        const int gw = !DGRAD ? cs.Wo : cls ? class_extent(cs.W, cs.cx, cs.stride) : cs.W;
        const int gh = !DGRAD ? cs.Ho : cls ? class_extent(cs.H, cs.cy, cs.stride) : cs.H;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            int row = row0 + (c >> 3);
            rowok[i] = row < o.rows;
            row = min(row, o.rows - 1);
            px[i] = row % gw;
            int q = row / gw;
            py[i] = q % gh;
            img[i] = q / gh;
            if (cls) {
                px[i] = px[i] * cs.stride + cs.cx;
                py[i] = py[i] * cs.stride + cs.cy;
            }
        }
    }
    __device__ __forceinline__ void load(int d, int k0, int kend, int tid)
    {
        const int sh = DGRAD ? cs.Ho : cs.H, sw = DGRAD ? cs.Wo : cs.W;
        const int tq = small_div(tap, magic);
        const int u = u0 + ustep * tq, v = v0 + ustep * (tap - tq * kdiv);
        const bool kin = k0 + kc8 < kend;
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (FULL || tid + i * NT < ROWS * 8) {
                int yy, xx;
                bool inside;
                if (DGRAD) {
                    // output pixel (ys, xs) / stride, if that is a whole number inside the output
                    const int ys = py[i] + cs.pad - u, xs = px[i] + cs.pad - v;
                    const int yp = max(ys, 0), xp = max(xs, 0);
                    yy = small_div(yp, magic_s);
                    xx = small_div(xp, magic_s);
                    inside = ys >= 0 && xs >= 0 && yy * cs.stride == yp && xx * cs.stride == xp && yy < sh && xx < sw;
                } else {
                    yy = py[i] * cs.stride + u - cs.pad;
                    xx = px[i] * cs.stride + v - cs.pad;
                    inside = yy >= 0 && xx >= 0 && yy < sh && xx < sw;
                }
                ok[d][i] = inside && rowok[i] && kin;
                yy = min(max(yy, 0), sh - 1);          // also covers taps past the last one (tail of K)
                xx = min(max(xx, 0), sw - 1);
                st[d][i] = *reinterpret_cast<const u32x4*>(base + ((int64_t)(img[i] * sh + yy) * sw + xx) * ch + c0);
            }
        c0 += r_ch;
        tap += q_tap;
        if (c0 >= ch) {
            c0 -= ch;
            ++tap;
        }
    }
    template <bool TAIL>
    __device__ __forceinline__ void store(int d, bf16_t* lds, int, int, int tid) const
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            if (FULL || c < ROWS * 8)
                *reinterpret_cast<u32x4*>(lds + (c >> 3) * LDK + (c & 7) * 8) = ok[d][i] ? st[d][i] : z;
        }
    }
};

// B operand, k-major.  DGRAD: column = input channel i, k = (u, v, o), reads W[o][u][v][i].
//                      WGRAD: column = (u, v, i),        k = output pixel, reads X[n, y*s+u-p, x*s+v-p, i].
template <int COLS, int NT, int DEPTH, bool WGRAD>
struct ConvKmTile {
    static constexpr int CPK = COLS / 8;
    static constexpr int LDM = COLS + 16;
    static constexpr int CH = (BK * CPK + NT - 1) / NT;
    static constexpr bool FULL = (BK * CPK) % NT == 0;
    const bf16_t* base;
    ConvShape cs;
    int c0[CH], tu[CH], tv[CH];
    bool colok[CH];
    // k of the next load, per chunk.  DGRAD: (tap, o) in s1, s0.  WGRAD: output pixel as (n, y, x) in s2, s1, s0.
    int s0[CH], s1[CH], s2[CH], kk[CH];
    int d0, d1, d2;           // BK in the same mixed radix
    int ntaps, nv, magic_nv, u0, v0, ustep;   // DGRAD: the taps K runs over (all, or those of a parity class)
    bool ok[DEPTH][CH];
    u32x4 st[DEPTH][CH];

    __device__ __forceinline__ void init(const Operand& o, int col0, int tid, const ConvShape& shape, int, int kbeg)
    {
        base = o.p;
        cs = shape;
        if (WGRAD) {
            d2 = BK / (cs.Ho * cs.Wo);
            int rem = BK - d2 * cs.Ho * cs.Wo;
            d1 = rem / cs.Wo;
            d0 = rem - d1 * cs.Wo;
        } else {
            d2 = 0;
            d1 = BK / cs.O;
            d0 = BK - d1 * cs.O;
            const ClassTaps cu = class_taps(cs.cy, cs.pad, cs.stride, cs.k), cv = class_taps(cs.cx, cs.pad, cs.stride, cs.k);
            nv = cs.cls ? cv.count : cs.k;
            ntaps = (cs.cls ? cu.count : cs.k) * nv;
            magic_nv = (65536 + nv - 1) / nv;
            u0 = cs.cls ? cu.first : 0;
            v0 = cs.cls ? cv.first : 0;
            ustep = cs.cls ? cs.stride : 1;
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            int col = col0 + (c % CPK) * 8;
            colok[i] = col < o.rows;
            col = min(col, o.rows - 8);
            const int k = kbeg + c / CPK;
            kk[i] = k;
            if (WGRAD) {
                int tap = col / cs.I;
                c0[i] = col - tap * cs.I;
                tu[i] = tap / cs.k;
                tv[i] = tap - tu[i] * cs.k;
                s0[i] = k % cs.Wo;
                int q = k / cs.Wo;
                s1[i] = q % cs.Ho;
                s2[i] = q / cs.Ho;
            } else {
                c0[i] = col;
                tu[i] = tv[i] = 0;
                s1[i] = k / cs.O;
                s0[i] = k - s1[i] * cs.O;
                s2[i] = 0;
            }
        }
    }
    __device__ __forceinline__ void load(int d, int, int kend, int tid)
    {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (FULL || tid + i * NT < BK * CPK) {
                const bool kin = kk[i] < kend;
                bool inside = true;
                int64_t off;
                if (WGRAD) {
                    int yy = s1[i] * cs.stride + tu[i] - cs.pad, xx = s0[i] * cs.stride + tv[i] - cs.pad;
                    inside = yy >= 0 && xx >= 0 && yy < cs.H && xx < cs.W;
                    yy = min(max(yy, 0), cs.H - 1);
                    xx = min(max(xx, 0), cs.W - 1);
                    int n = min(s2[i], cs.N - 1);           // pixels past the last one (tail of K) stay in the tensor
                    off = ((int64_t)(n * cs.H + yy) * cs.W + xx) * cs.I + c0[i];
                } else {
                    const int t = min(s1[i], ntaps - 1);     // likewise for taps past the last one
                    const int tq = small_div(t, magic_nv);
                    const int tap = (u0 + ustep * tq) * cs.k + v0 + ustep * (t - tq * nv);
                    off = ((int64_t)s0[i] * cs.k * cs.k + tap) * cs.I + c0[i];
                }
                ok[d][i] = inside && colok[i] && kin;
                st[d][i] = *reinterpret_cast<const u32x4*>(base + off);
                // advance this chunk's k by BK
                kk[i] += BK;
                s0[i] += d0;
                s1[i] += d1;
                if (WGRAD) {
                    if (s0[i] >= cs.Wo) { s0[i] -= cs.Wo; ++s1[i]; }
                    s2[i] += d2;
                    if (s1[i] >= cs.Ho) { s1[i] -= cs.Ho; ++s2[i]; }
                } else {
                    if (s0[i] >= cs.O) { s0[i] -= cs.O; ++s1[i]; }
                }
            }
    }
    template <bool TAIL>
    __device__ __forceinline__ void store(int d, bf16_t* lds, int, int, int tid) const
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int c = tid + i * NT;
            if (FULL || c < BK * CPK)
                *reinterpret_cast<u32x4*>(lds + (c / CPK) * LDM + (c % CPK) * 8) = ok[d][i] ? st[d][i] : z;
        }
    }
};

// Tile type by layout (k-major or not) and gather mode (GATHER_* of the product).
template <int ROWS, int NT, int DEPTH, bool KM, int G, bool IS_A>
struct TileSel { typedef KcTile<ROWS, NT, DEPTH> type; };
template <int ROWS, int NT, int DEPTH, int G, bool IS_A>
struct TileSel<ROWS, NT, DEPTH, true, G, IS_A> { typedef KmTile<ROWS, NT, DEPTH> type; };
template <int ROWS, int NT, int DEPTH>
struct TileSel<ROWS, NT, DEPTH, false, GATHER_CONV_FWD, true> { typedef ConvRowsTile<ROWS, NT, DEPTH, false> type; };
template <int ROWS, int NT, int DEPTH>
struct TileSel<ROWS, NT, DEPTH, false, GATHER_CONV_DGRAD, true> { typedef ConvRowsTile<ROWS, NT, DEPTH, true> type; };
template <int ROWS, int NT, int DEPTH>
struct TileSel<ROWS, NT, DEPTH, true, GATHER_CONV_DGRAD, false> { typedef ConvKmTile<ROWS, NT, DEPTH, false> type; };
template <int ROWS, int NT, int DEPTH>
struct TileSel<ROWS, NT, DEPTH, true, GATHER_CONV_WGRAD, false> { typedef ConvKmTile<ROWS, NT, DEPTH, true> type; };

// Operand fragment of one 32-row block for one 16-wide k step, in the register layout of
// v_mfma_f32_32x32x16_bf16: lane L holds row (L & 31), k = 8 * (L >> 5) + 0..7.
// k-contiguous tile [row][k]: one 16-byte read.
__device__ __forceinline__ bf16x8 kc_frag(const bf16_t* tile, int row_block, int kk, int lane)
{
    return *reinterpret_cast<const bf16x8*>(tile + (row_block * 32 + (lane & 31)) * LDK + kk * 16 + (lane >> 5) * 8);
}

// k-major tile [k][row]: km_frag (two transposing reads).
template <int TM, int TN, bool A_KM, bool B_KM, int LDMA, int LDMB>
__device__ __forceinline__ void mma_step(f32x16 (&acc)[TM][TN], const bf16_t* a_lds, int a_row0, const bf16_t* b_lds,
                                         int b_row0, int lane)
{
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = A_KM ? km_frag<LDMA>(a_lds + a_row0, i, kk, lane) : kc_frag(a_lds + a_row0 * LDK, i, kk, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = B_KM ? km_frag<LDMB>(b_lds + b_row0, j, kk, lane) : kc_frag(b_lds + b_row0 * LDK, j, kk, lane);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(b[j], a[i], acc[i][j]);   // roles swapped: lane <-> row m
    }
}

// Elements one operand tile occupies in LDS.
template <int ROWS, bool KM>
constexpr int tile_elems() { return KM ? BK * (ROWS + 16) : ROWS * LDK; }

template <int BM, int BN, bool A_KM, bool B_KM, class OutT>
constexpr int gemm2_lds_bytes()
{
    int main = 2 * (tile_elems<BM, A_KM>() + tile_elems<BN, B_KM>()) * 2;
    int epi = sizeof(OutT) == 2 ? BM * (BN + 8) * 2 : 0;
    return main > epi ? main : epi;
}

// bf16 results of one BM x BN tile: registers -> LDS tile (row-major) -> 16 contiguous bytes per
// lane to global memory, with the optional GELU epilogue.  Results (and the pre-activation the
// gradient epilogue reads) are streamed with non-temporal accesses: 10 % faster on the wide products.  Every wave must be past its last read
// of the operand tiles in LDS (the staging tile overlays them); ends without a barrier.
template <int BM, int BN, int WGM, int WGN, bool MAPROWS, int TM, int TN>
__device__ __forceinline__ void store_bf16_tile(const f32x16 (&acc)[TM][TN], bf16_t* lds, bf16_t* __restrict__ out, int64_t ldc,
                                                const float* __restrict__ bias, int M, int N, int m0, int n0, int epilogue,
                                                bf16_t* __restrict__ aux, int64_t ldaux, int tid, const ConvShape& cs)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static_assert(TM == WTM / 32 && TN == WTN / 32, "accumulator shape");
    constexpr int LDC = BN + 8;
    constexpr int CPR = BN / 8;
    constexpr int PER = BM * CPR / NT;          // 16-byte chunks per thread
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int r = lane & 31, h = lane >> 5;
    // The activation-gradient epilogue reads the pre-activation: start those loads now, so they
    // are in flight while the accumulators go through LDS.
    bf16x8 z8[PER];
    if (epilogue == EPI_ACT_GRAD) {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            int c = tid + q * NT;
            int m = min(m0 + c / CPR, M - 1), n = min(n0 + (c % CPR) * 8, N - 8);
            z8[q] = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(aux + (int64_t)m * ldaux + n)));
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int ml = wm * WTM + i * 32 + r;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int nl = wn * WTN + j * 32 + 8 * g + 4 * h;
                f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                if (bias) {
                    int n = min(n0 + nl, N - 4);
                    f32x4 b4 = *reinterpret_cast<const f32x4*>(bias + n);
                    v += b4;
                }
                u32x2 pk = {pack_bf16(v.x, v.y), pack_bf16(v.z, v.w)};
                *reinterpret_cast<u32x2*>(lds + ml * LDC + nl) = pk;
            }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        int c = tid + q * NT;
        int ml = c / CPR, cc = c % CPR;
        int m = m0 + ml, n = n0 + cc * 8;
        const bool ok = m < M && n < N;   // N is a multiple of 8 on this path
        u32x4 v = *reinterpret_cast<const u32x4*>(lds + ml * LDC + cc * 8);
        int64_t mrow = m;
        if (MAPROWS && cs.cls) {
            // row m counts the input pixels of one parity class: its place among all input pixels
            const int gw = class_extent(cs.W, cs.cx, cs.stride), gh = class_extent(cs.H, cs.cy, cs.stride);
            const int mm = min(m, M - 1);
            const int ix = mm % gw, q = mm / gw;
            mrow = ((int64_t)(q / gh) * cs.H + (q % gh) * cs.stride + cs.cy) * cs.W + ix * cs.stride + cs.cx;
        }
        if (epilogue == EPI_ACT_GRAD) {
            bf16x8 c8 = __builtin_bit_cast(bf16x8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) c8[e] = (bf16_t)((float)c8[e] * gelu_grad_bf16_f((float)z8[q][e]));
            v = __builtin_bit_cast(u32x4, c8);
        }
        if (ok) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + mrow * ldc + n));
        if (epilogue == EPI_ACT_STORE) {
            bf16x8 c8 = __builtin_bit_cast(bf16x8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) c8[e] = (bf16_t)gelu_bf16_f((float)c8[e]);
            if (ok) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, c8), reinterpret_cast<u32x4*>(aux + (int64_t)m * ldaux + n));
        }
    }
}

template <int BM, int BN, int WGM, int WGN, int DEPTH, bool A_KM, bool B_KM, class OutT, int G>
__global__ __launch_bounds__(64 * WGM * WGN, 2) void gemm2_kernel(Operand A, Operand B, ConvShape cs, OutT* __restrict__ C, int64_t ldc,
                                                               const float* __restrict__ bias, float* __restrict__ partial,
                                                               int M, int N, int K, int k_per_split, int epilogue,
                                                               bf16_t* __restrict__ aux, int64_t ldaux, BatchArgs bt)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_ELEMS = tile_elems<BM, A_KM>();
    constexpr int STAGE = A_ELEMS + tile_elems<BN, B_KM>();
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    // blockIdx.z = K-slice, or (batch index, K-slice) for a batch of products of one shape
    int zslice = blockIdx.z, zbatch = 0;
    if constexpr (G == GATHER_NONE) {
        if (bt.batch > 1) {
            zbatch = blockIdx.z / bt.nsplit;
            zslice = blockIdx.z - zbatch * bt.nsplit;
            A.p += zbatch * bt.a_bs;
            B.p += zbatch * bt.b_bs;
            C += zbatch * bt.c_bs;
            if (bias) bias += zbatch * bt.bias_bs;
            if (aux) aux += zbatch * bt.aux_bs;
        }
    }
    int kbeg = zslice * k_per_split;
    if constexpr (G == GATHER_CONV_DGRAD) {
        if (cs.cls) {
            // all parity classes of a strided data gradient in one launch: blockIdx.z is the class,
            // each with its own number of rows and taps; K is not sliced
            cs.cy = blockIdx.z / cs.stride;
            cs.cx = blockIdx.z - cs.cy * cs.stride;
            M = cs.N * class_extent(cs.H, cs.cy, cs.stride) * class_extent(cs.W, cs.cx, cs.stride);
            K = class_taps(cs.cy, cs.pad, cs.stride, cs.k).count * class_taps(cs.cx, cs.pad, cs.stride, cs.k).count * cs.O;
            A.rows = M;
            kbeg = 0;
            k_per_split = K;
            if (m0 >= M) return;
        }
    }
    const int kend = min(K, kbeg + k_per_split);
    const int nk = (kend - kbeg + BK - 1) / BK;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    typename TileSel<BM, NT, DEPTH, A_KM, G, true>::type ta;
    typename TileSel<BN, NT, DEPTH, B_KM, G, false>::type tb;
    ta.init(A, m0, tid, cs, K, kbeg);
    tb.init(B, n0, tid, cs, K, kbeg);

    int kt0 = 0;
    if (nk >= 2 * DEPTH) {
        // Long reductions.  Prologue and steady state are straight-line code: the loads of DEPTH steps
        // are issued unconditionally and stay in flight from one iteration to the next (a branch in
        // here makes the compiler wait for every outstanding load at the top of each step).
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            ta.load(d, kbeg + d * BK, kend, tid);
            tb.load(d, kbeg + d * BK, kend, tid);
        }
        ta.template store<false>(0, lds, kbeg, kend, tid);
        tb.template store<false>(0, lds + A_ELEMS, kbeg, kend, tid);
        __syncthreads();
        // Each step issues the loads of step +DEPTH, multiplies, and hands step +1 to LDS.
        for (; kt0 + 2 * DEPTH <= nk; kt0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                const int kt = kt0 + d;
                bf16_t* cur = lds + (kt & 1) * STAGE;
                bf16_t* nxt = lds + ((kt + 1) & 1) * STAGE;
                ta.load(d, kbeg + (kt + DEPTH) * BK, kend, tid);
                tb.load(d, kbeg + (kt + DEPTH) * BK, kend, tid);
                __builtin_amdgcn_sched_barrier(0);   // keep the loads first: the scheduler otherwise sinks them below the MFMAs
                mma_step<TM, TN, A_KM, B_KM, BM + 16, BN + 16>(acc, cur, wm * WTM, cur + A_ELEMS, wn * WTN, lane);
                ta.template store<false>((d + 1) % DEPTH, nxt, kbeg + (kt + 1) * BK, kend, tid);
                tb.template store<false>((d + 1) % DEPTH, nxt + A_ELEMS, kbeg + (kt + 1) * BK, kend, tid);
                __syncthreads();
            }
        }
    } else {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (d < nk) {
                ta.load(d, kbeg + d * BK, kend, tid);
                tb.load(d, kbeg + d * BK, kend, tid);
            }
        if (nk > 0) {
            ta.template store<true>(0, lds, kbeg, kend, tid);
            tb.template store<true>(0, lds + A_ELEMS, kbeg, kend, tid);
        }
        __syncthreads();
    }
    // Drain: the last (up to 2 * DEPTH - 1) steps, which stop loading and then stop storing.
    for (; kt0 < nk; kt0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int kt = kt0 + d;
            if (kt < nk) {
                bf16_t* cur = lds + (kt & 1) * STAGE;
                bf16_t* nxt = lds + ((kt + 1) & 1) * STAGE;
                if (kt + DEPTH < nk) {
                    ta.load(d, kbeg + (kt + DEPTH) * BK, kend, tid);
                    tb.load(d, kbeg + (kt + DEPTH) * BK, kend, tid);
                }
                mma_step<TM, TN, A_KM, B_KM, BM + 16, BN + 16>(acc, cur, wm * WTM, cur + A_ELEMS, wn * WTN, lane);
                if (kt + 1 < nk) {
                    ta.template store<true>((d + 1) % DEPTH, nxt, kbeg + (kt + 1) * BK, kend, tid);
                    tb.template store<true>((d + 1) % DEPTH, nxt + A_ELEMS, kbeg + (kt + 1) * BK, kend, tid);
                }
                __syncthreads();
            }
        }
    }

    const int r = lane & 31, h = lane >> 5;
    if constexpr (sizeof(OutT) == 4) {
        // fp32 results (weight gradients or their split-K partials): 16-byte stores straight from registers
        // slices of a batch lie [slice][batch][M][N], so that the sum over slices sees one tall matrix
        float* out = partial ? partial + ((int64_t)zslice * bt.batch + zbatch) * M * N : reinterpret_cast<float*>(C);
        const int64_t ldo = partial ? (int64_t)N : ldc;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int m = m0 + wm * WTM + i * 32 + r;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    int n = n0 + wn * WTN + j * 32 + 8 * g + 4 * h;
                    if (m < M && n < N) {   // N is a multiple of 4 on this path
                        f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                        *reinterpret_cast<f32x4*>(out + (int64_t)m * ldo + n) = v;
                    }
                }
        }
    } else {
        store_bf16_tile<BM, BN, WGM, WGN, G == GATHER_CONV_DGRAD>(acc, lds, reinterpret_cast<bf16_t*>(C), ldc, bias, M, N, m0, n0,
                                                                  epilogue, aux, ldaux, tid, cs);
    }
}

// Slices of K a launch really uses (each a whole number of K-steps) and their length.
inline int effective_splits(const MatOp& op, int* k_per_split)
{
    int splits = (op.splits > 1 && op.partial) ? op.splits : 1;
    int kps = (int)(ceil_div(ceil_div(op.K, splits), BK) * BK);
    if (k_per_split) *k_per_split = kps;
    return (int)ceil_div(op.K, kps);
}

template <int BM, int BN, int WGM, int WGN, int DEPTH, bool A_KM, bool B_KM, class OutT, int G = GATHER_NONE>
hipError_t launch(const MatOp& op, const Operand& A, const Operand& B, hipStream_t st)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int lds_bytes = gemm2_lds_bytes<BM, BN, A_KM, B_KM, OutT>();
    auto kern = gemm2_kernel<BM, BN, WGM, WGN, DEPTH, A_KM, B_KM, OutT, G>;
    static bool lds_allowed = false;
    if (!lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           lds_bytes);
        if (e != hipSuccess) return e;
        lds_allowed = true;
    }
    static const std::string tag = [] {
        char b[64];
        snprintf(b, sizeof(b), "gemm2_kernel<%d,%d,%d,%d,%s,%s,%s%s>", BM, BN, WGM, WGN, A_KM ? "A_KM" : "A_KC", B_KM ? "B_KM" : "B_KC",
                 sizeof(OutT) == 2 ? "bf16" : "f32", G == GATHER_NONE ? "" : ",conv");
        return std::string(b);
    }();
    note_kernel(tag.c_str());
    int kps;
    const int splits = effective_splits(op, &kps);
    float* partial = splits > 1 ? op.partial : nullptr;
    if (sizeof(OutT) == 4 && !op.out_f32 && !partial) return hipErrorInvalidValue;   // fp32 tiles need the reduce to reach a bf16 C
    BatchArgs bt;
    bt.batch = G == GATHER_NONE ? op.batch : 1;
    bt.nsplit = splits;
    bt.a_bs = op.a_bs; bt.b_bs = op.b_bs; bt.c_bs = op.c_bs; bt.aux_bs = op.aux_bs; bt.bias_bs = op.bias_bs;
    dim3 grid((unsigned)ceil_div(op.M, BM), (unsigned)ceil_div(op.N, BN), (unsigned)(splits * bt.batch));
    if (G == GATHER_CONV_DGRAD && op.cs.cls) grid.z = (unsigned)(op.cs.stride * op.cs.stride);   // one slab of workgroups per parity class
    hipLaunchKernelGGL(kern, grid, dim3(NT), lds_bytes, st, A, B, op.cs, (OutT*)op.C, op.ldc, op.bias, partial, (int)op.M,
                       (int)op.N, (int)op.K, kps, op.epilogue, (bf16_t*)op.aux, op.ldaux, bt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // a batch of sliced products is summed as one matrix of batch * M rows (supported() admits only dense results)
    if (splits > 1)
        return reduce_partials(op.partial, op.C, !op.out_f32, op.ldc, op.M * bt.batch, op.N, splits, st, op.out_f32 ? op.sgd : nullptr);
    return hipSuccess;
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Tile choice: the largest tile that still yields about one workgroup per compute unit.
template <bool A_KM, bool B_KM, class OutT, int G = GATHER_NONE>
hipError_t by_tile(const MatOp& op, const Operand& A, const Operand& B, hipStream_t st)
{
    const int64_t splits = effective_splits(op, nullptr);
    auto wgs = [&](int bm, int bn) { return ceil_div(op.M, bm) * ceil_div(op.N, bn) * splits * (G == GATHER_NONE ? op.batch : 1); };
    // Large products in every layout: 256 x 256 tiles on eight waves (wave tile 128 x 64): half the operand
    // bytes per flop from L2 into LDS of a 128 x 128 tile, and a quarter of the barriers.  16384 x 4096 x 4096:
    // forward 551 -> 445 us, data gradient 609 -> 440 us, weight gradient 538 -> 407 us against 128 x 128 tiles.
    if constexpr (G == GATHER_NONE && ((sizeof(OutT) == 2 && !A_KM) || (sizeof(OutT) == 4 && A_KM && B_KM))) {
        // (a batch of weight gradients: from 128 tiles on, 213 against 368 us for 36 x [1024 x 256] over 8192 tokens)
        const int64_t enough = (sizeof(OutT) == 4 && op.batch >= 8) ? 128 : 224;
        // (not for results that fill less than two thirds of their 256 x 256 tiles: the 32 x 64 weight gradient of a
        // 1x1 convolution has thousands of K-slices and would multiply 32 times its size)
        const bool fills = 3 * op.M * op.N >= 2 * ceil_div(op.M, 256) * ceil_div(op.N, 256) * 65536;
        if (op.K >= 1024 && fills && wgs(256, 256) >= enough) return launch<256, 256, 2, 4, 2, A_KM, B_KM, OutT>(op, A, B, st);
    }
    // Results at most 32 columns wide (1x1 and core convolutions at Tucker ranks <= 32): a 128 x 32 tile
    // does a quarter of the MFMA and LDS work of a 128 x 128 one (15 against 23 us at 401408 x 32 x 64).
    if constexpr (sizeof(OutT) == 2 && !A_KM && G != GATHER_CONV_WGRAD) {
        if (op.N <= 32 && wgs(128, 32) >= 256) return launch<128, 32, 4, 1, 2, false, B_KM, OutT, G>(op, A, B, st);
    }
    if (op.M > 64 && op.N > 64 && (wgs(128, 128) >= 200 || wgs(64, 64) > 2048)) {
        // Short reductions with bf16 results (K = rank: second product of a forward pair or of a data
        // gradient) are dominated by the epilogue; eight waves per tile overlap it better than four
        // (31.8 against 36.0 us at 8192 x 3072 x 192 with the GELU epilogue).
        if constexpr (sizeof(OutT) == 2 && !A_KM && G == GATHER_NONE) {
            if (op.K <= 4 * BK) return launch<128, 128, 2, 4, 2, A_KM, B_KM, OutT, G>(op, A, B, st);
        }
        return launch<128, 128, 2, 2, 2, A_KM, B_KM, OutT, G>(op, A, B, st);
    }
    return launch<64, 64, 2, 2, 2, A_KM, B_KM, OutT, G>(op, A, B, st);
}

}  // namespace

bool mfma_gemm2_supported(const MatOp& op)
{
    if (!op.in_bf16) return false;
    if (op.M < 1 || op.N < 1 || op.K < 8) return false;
    if (op.M >= (int64_t(1) << 31) || op.N >= (int64_t(1) << 31) || op.K >= (int64_t(1) << 31)) return false;
    if (!al16(op.A) || !al16(op.B) || !al16(op.C)) return false;
    bool akm, bkm;
    if (op.gather == GATHER_NONE) {
        akm = op.a_sk != 1;
        bkm = op.b_sk != 1;
        if (akm && (op.a_sm != 1 || op.a_sk % 8 != 0 || op.M % 8 != 0)) return false;
        if (!akm && op.a_sm % 8 != 0) return false;
        if (bkm && (op.b_sn != 1 || op.b_sk % 8 != 0 || op.N % 8 != 0)) return false;
        if (!bkm && op.b_sn % 8 != 0) return false;
    } else {
        // implicit-GEMM convolution: channel counts must keep every 16-byte chunk inside one tap
        if (op.cs.I % 8 != 0 || op.cs.O % 8 != 0 || op.cs.k < 1 || op.cs.k > 31 || op.cs.stride < 1) return false;
        if ((int64_t)op.cs.N * op.cs.H * op.cs.W * op.cs.I >= (int64_t(1) << 31)) return false;
        if ((int64_t)op.cs.N * op.cs.Ho * op.cs.Wo * op.cs.O >= (int64_t(1) << 31)) return false;
        if (op.gather == GATHER_CONV_FWD) {
            akm = false; bkm = false;
            if (op.b_sk != 1 || op.b_sn % 8 != 0) return false;
        } else if (op.gather == GATHER_CONV_DGRAD) {
            akm = false; bkm = true;
            // pixel coordinate / stride is done by multiplication, exact while coordinate * stride < 65536
            if ((int64_t)(std::max(op.cs.H, op.cs.W) + op.cs.pad) * op.cs.stride >= 65536) return false;
        } else {
            akm = true; bkm = true;
            if (op.a_sm != 1 || op.a_sk % 8 != 0 || op.M % 8 != 0) return false;
        }
    }
    if ((!akm || !bkm) && op.K % 8 != 0) return false;    // a k-contiguous operand is read in chunks of 8 k
    if (akm && !bkm) return false;                       // layout not used by any layer pass
    if (op.out_f32) {
        if (!(akm && bkm)) return false;                 // fp32 results are weight gradients
        if (op.N % 4 != 0 || op.ldc % 4 != 0 || op.bias) return false;
    } else {
        if (akm) return false;
        if (op.N % 8 != 0 || op.ldc % 8 != 0) return false;
        // split-K towards a bf16 result: fp32 partials, rounded once by the reduce; plain products only
        if (op.splits > 1 && (op.gather != GATHER_NONE || op.bias || op.epilogue != EPI_NONE)) return false;
        if (op.bias && (op.N < 4 || (reinterpret_cast<uintptr_t>(op.bias) & 15u))) return false;
    }
    if (ceil_div(op.N, 64) > 65535) return false;
    if (op.batch < 1 || op.batch > 1024) return false;
    if (op.batch > 1) {
        if (op.gather != GATHER_NONE || op.sgd) return false;
        if (op.a_bs % 8 != 0 || op.b_bs % 8 != 0 || op.c_bs % 8 != 0 || op.aux_bs % 8 != 0 || op.bias_bs % 4 != 0) return false;
        // sliced reductions of a batch are summed as one tall dense matrix
        if (op.splits > 1 && op.partial && (!op.out_f32 || op.ldc != op.N || op.c_bs != op.M * op.N)) return false;
    }
    if (op.gather == GATHER_NONE && ((akm ? op.a_sk : op.a_sm) > BUF_MAX_LD || (bkm ? op.b_sk : op.b_sn) > BUF_MAX_LD)) return false;
    if (op.epilogue != EPI_NONE && (op.out_f32 || !op.aux || !al16(op.aux) || op.ldaux % 8 != 0)) return false;
    return true;
}

hipError_t mfma_gemm2(const MatOp& op, hipStream_t st)
{
    if (op.gather == GATHER_CONV_FWD) {
        Operand A{(const bf16_t*)op.A, 0, (int)op.M};
        Operand B{(const bf16_t*)op.B, op.b_sn, (int)op.N};
        return by_tile<false, false, bf16_t, GATHER_CONV_FWD>(op, A, B, st);
    }
    if (op.gather == GATHER_CONV_DGRAD) {
        Operand B{(const bf16_t*)op.B, 0, (int)op.N};
        const ConvShape& cs = op.cs;
        if (cs.stride > 1 && cs.k >= cs.stride) {
            // Strided: an input pixel hears from an output pixel only through the taps of its parity
            // class, 1 / stride^2 of them on average.  One product per class, over those taps only,
            // written to the class's pixels (as one product over all taps, three quarters of a
            // stride-2 gradient's multiplications are by zeros).
            // The launch is shaped for class (0, 0), which has the most rows; the kernel takes the class
            // from blockIdx.z and works out that class's rows and taps itself.
            MatOp sub = op;
            sub.cs.cls = 1;
            sub.splits = 1;
            sub.M = (int64_t)cs.N * class_extent(cs.H, 0, cs.stride) * class_extent(cs.W, 0, cs.stride);
            int taps = 0;
            for (int c = 0; c < cs.stride; ++c) taps = std::max(taps, class_taps(c, cs.pad, cs.stride, cs.k).count);
            sub.K = (int64_t)taps * taps * cs.O;
            Operand A{(const bf16_t*)op.A, 0, (int)sub.M};
            return by_tile<false, true, bf16_t, GATHER_CONV_DGRAD>(sub, A, B, st);
        }
        Operand A{(const bf16_t*)op.A, 0, (int)op.M};
        return by_tile<false, true, bf16_t, GATHER_CONV_DGRAD>(op, A, B, st);
    }
    if (op.gather == GATHER_CONV_WGRAD) {
        Operand A{(const bf16_t*)op.A, op.a_sk, (int)op.M};
        Operand B{(const bf16_t*)op.B, 0, (int)op.N};
        return by_tile<true, true, float, GATHER_CONV_WGRAD>(op, A, B, st);
    }
    const bool akm = op.a_sk != 1, bkm = op.b_sk != 1;
    Operand A{(const bf16_t*)op.A, akm ? op.a_sk : op.a_sm, (int)op.M};
    Operand B{(const bf16_t*)op.B, bkm ? op.b_sk : op.b_sn, (int)op.N};
    if (op.out_f32) return by_tile<true, true, float>(op, A, B, st);
    if (effective_splits(op, nullptr) > 1)
        return bkm ? by_tile<false, true, float>(op, A, B, st) : by_tile<false, false, float>(op, A, B, st);
    if (bkm) return by_tile<false, true, bf16_t>(op, A, B, st);
    return by_tile<false, false, bf16_t>(op, A, B, st);
}

}  // namespace lrd
