// 3 x 3, stride 1 convolution on NHWC bf16 data for small channel counts (32 or 64 in and out): the
// core layer of a Tucker-decomposed convolution at the early stages of a ResNet, where the ranks are
// small and the images large.  Forward, data gradient and weight gradient.
//
// As an implicit GEMM such a layer fetches every input pixel nine times from L2 (once per tap) for
// very little arithmetic.  Here a workgroup stages an (8 + 2) x (32 + 2) pixel patch of the input in
// LDS once and forms the MFMA operand of every tap by reading the patch at a shifted position, so
// global traffic is the patch (1.3x the tile) and there are a few barriers per tile instead of one
// per K-step.  A workgroup walks over a run of tiles and has the next tile's data on its way into
// registers while it multiplies the current one.
//
// Forward: the weights sit in LDS next to the patch; each of the four waves owns two output rows of
// 32 pixels, and a weight fragment read from LDS is used for both.
// Data gradient: the same convolution of dY with the taps flipped, the channel roles exchanged and
// padding 2 - pad.  The weights are staged as they are; the exchange of roles is done by reading
// their fragments with the transposing LDS read.
// Weight gradient: dW[o][t][i] = sum over pixels of dY[pixel][o] * X[pixel + t][i].  The pixels are
// the contraction index, so both fragments come out of [pixel][channel] tiles by transposing reads;
// a wave keeps the accumulators of all nine taps of one channel-block pair and builds the three
// horizontally shifted fragments of a patch row from one read.  Each workgroup writes one fp32
// partial, summed afterwards in a fixed order.
#include <algorithm>

#include "lrd_internal.hpp"

namespace lrd {
namespace {

constexpr int TH = 8, TW = 32;           // output pixels per workgroup tile
constexpr int PH = TH + 2, PW = TW + 2;  // input patch
constexpr int NTHREADS = 256;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// A RH x RW pixel rectangle of an [N][Hh][Ww][C] tensor on its way from global memory to LDS
// ([pixel][C + 8] elements), held in registers in between.  Every load is in bounds (clamped);
// pixels outside the image are marked in `inside` and become zeros when the registers go to LDS,
// so that nothing waits for the loads before that.
template <int RH, int RW, int C>
struct Rect {
    static constexpr int CP = C / 8;                              // 16-byte chunks per pixel
    static constexpr int CHUNKS = RH * RW * CP;
    static constexpr int PER = (CHUNKS + NTHREADS - 1) / NTHREADS;
    static constexpr int LD = C + 8;                              // LDS elements per pixel: conflict-free fragment reads
    u32x4 v[PER];
    uint32_t inside;

    __device__ __forceinline__ void fetch(const bf16_t* __restrict__ img, int Hh, int Ww, int ybase, int xbase, int tid)
    {
        inside = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = min(tid + NTHREADS * i, CHUNKS - 1);
            const int pix = c / CP, c8 = (c - pix * CP) * 8;
            const int py = pix / RW, px = pix - py * RW;
            const int iy = ybase + py, ix = xbase + px;
            const int cy = min(max(iy, 0), Hh - 1), cx = min(max(ix, 0), Ww - 1);
            v[i] = *reinterpret_cast<const u32x4*>(img + ((int64_t)cy * Ww + cx) * C + c8);
            inside |= (iy == cy && ix == cx) ? (1u << i) : 0u;
        }
    }
    __device__ __forceinline__ void to_lds(bf16_t* lds, int tid) const
    {
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + NTHREADS * i;
            const int pix = c / CP, c8 = (c - pix * CP) * 8;
            if (c < CHUNKS) *reinterpret_cast<u32x4*>(lds + pix * LD + c8) = ((inside >> i) & 1u) ? v[i] : zero;
        }
    }
};

struct TileAt { int n, y0, x0; };
__device__ __forceinline__ TileAt tile_at(int tile, int tiles_x, int tiles_y)
{
    const int tx = tile % tiles_x, rest = tile / tiles_x;
    return {rest / tiles_y, (rest % tiles_y) * TH, tx * TW};
}

// ------------------------------------------------------------------------- forward / data gradient
// LDS elements of the patch region; the finished output tile is staged there too.
template <int CI, int CO>
constexpr int patch_elems() { return PH * PW * (CI + 8) > TH * TW * (CO + 8) ? PH * PW * (CI + 8) : TH * TW * (CO + 8); }
// Weights in LDS: [CO][9 CI + 8], or, for the data gradient (WT), [CI][9 CO + 8] as they lie in memory.
template <int CI, int CO, bool WT>
constexpr int weight_ld() { return 9 * (WT ? CO : CI) + 8; }
template <int CI, int CO, bool WT>
constexpr int conv_lds_bytes() { return (patch_elems<CI, CO>() + (WT ? CI : CO) * weight_ld<CI, CO, WT>()) * 2; }

// out[n][y][x][co] = sum over taps t = (u, v) and ci of in[n][y + u - pad][x + v - pad][ci] * W(co, t, ci)
// with W(co, t, ci) = w[co][t][ci], or w[ci][8 - t][co] when WT.  in [N][Hi][Wi][CI], out [N][Ho][Wo][CO].
// Workgroup b computes tiles b * tiles_per_wg ... of ntiles = N * tiles_y * tiles_x (x fastest).
template <int CI, int CO, bool WT>
__global__ __launch_bounds__(NTHREADS) void conv3x3_direct_kernel(const bf16_t* __restrict__ in, const bf16_t* __restrict__ w,
                                                                  bf16_t* __restrict__ out, int Hi, int Wi, int Ho, int Wo, int pad,
                                                                  int tiles_x, int tiles_y, int ntiles, int tiles_per_wg)
{
    typedef Rect<PH, PW, CI> Patch;
    constexpr int PS = Patch::LD;
    constexpr int WS = weight_ld<CI, CO, WT>();
    constexpr int OS = CO + 8;            // LDS elements per staged output pixel
    constexpr int CPO = CO / 8;           // 16-byte chunks per output pixel
    constexpr int NB = CO / 32;           // 32-wide blocks of output channels
    constexpr int KK = CI / 16;           // MFMA K-steps per tap
    constexpr int W_ROW_CHUNKS = (WS - 8) / 8, W_CHUNKS = (WT ? CI : CO) * W_ROW_CHUNKS;
    constexpr int NWI = (W_CHUNKS + NTHREADS - 1) / NTHREADS, NOI = TH * TW * CPO / NTHREADS;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* patch = reinterpret_cast<bf16_t*>(smem);
    bf16_t* wl = patch + patch_elems<CI, CO>();
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, h = lane >> 5, lk = h * 8;
    const int first = blockIdx.x * tiles_per_wg, last = min(first + tiles_per_wg, ntiles);

    Patch next;
    {
        u32x4 wv[NWI];
#pragma unroll
        for (int i = 0; i < NWI; ++i) wv[i] = *reinterpret_cast<const u32x4*>(w + (int64_t)min(tid + NTHREADS * i, W_CHUNKS - 1) * 8);
        const TileAt t0 = tile_at(first, tiles_x, tiles_y);
        next.fetch(in + (int64_t)t0.n * Hi * Wi * CI, Hi, Wi, t0.y0 - pad, t0.x0 - pad, tid);
#pragma unroll
        for (int i = 0; i < NWI; ++i) {
            const int c = tid + NTHREADS * i;
            const int row = c / W_ROW_CHUNKS, k8 = (c - row * W_ROW_CHUNKS) * 8;
            if (c < W_CHUNKS) *reinterpret_cast<u32x4*>(wl + row * WS + k8) = wv[i];
        }
    }

    for (int tile = first; tile < last; ++tile) {
        const TileAt at = tile_at(tile, tiles_x, tiles_y);
        next.to_lds(patch, tid);
        __syncthreads();
        if (tile + 1 < last) {
            const TileAt an = tile_at(tile + 1, tiles_x, tiles_y);
            next.fetch(in + (int64_t)an.n * Hi * Wi * CI, Hi, Wi, an.y0 - pad, an.x0 - pad, tid);
        }

        // wave `wave` computes tile rows 2 wave and 2 wave + 1, 32 pixels each; the fragments of
        // step s + 1 (tap, 16 channels) are read from LDS while step s is multiplied
        f32x16 acc[2][NB];
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[r][j][e] = 0.f;
        bf16x8 wf[2][NB], pf[2][2];
        auto read_frags = [&](int s, int buf) {
            const int t = s / KK, kk = s - t * KK;
            const int u = t / 3, v = t - u * 3;
#pragma unroll
            for (int j = 0; j < NB; ++j)
                wf[buf][j] = WT ? km_frag<WS>(wl + (8 - t) * CO, j, kk, lane)
                                : *reinterpret_cast<const bf16x8*>(wl + (j * 32 + lrow) * WS + t * CI + kk * 16 + lk);
#pragma unroll
            for (int r = 0; r < 2; ++r)
                pf[buf][r] = *reinterpret_cast<const bf16x8*>(patch + ((2 * wave + r + u) * PW + lrow + v) * PS + kk * 16 + lk);
        };
        read_frags(0, 0);
#pragma unroll
        for (int s = 0; s < 9 * KK; ++s) {
            if (s + 1 < 9 * KK) read_frags(s + 1, (s + 1) & 1);
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int j = 0; j < NB; ++j) acc[r][j] = mfma32(wf[s & 1][j], pf[s & 1][r], acc[r][j]);   // lane <-> pixel, values <-> channels
        }
        __syncthreads();   // every wave is done with the patch: the output tile is staged over it

        // lane holds, for its pixel, channels 8 g + 4 h + 0..3 of every 32-channel block
        bf16_t* stage = patch;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 pk = {pack_bf16(acc[r][j][4 * g], acc[r][j][4 * g + 1]), pack_bf16(acc[r][j][4 * g + 2], acc[r][j][4 * g + 3])};
                    *reinterpret_cast<u32x2*>(stage + ((2 * wave + r) * TW + lrow) * OS + j * 32 + 8 * g + 4 * h) = pk;
                }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < NOI; ++q) {
            const int c = tid + NTHREADS * q;
            const int pix = c / CPO, c8 = (c - pix * CPO) * 8;
            const int oy = at.y0 + pix / TW, ox = at.x0 + pix % TW;
            const u32x4 v = *reinterpret_cast<const u32x4*>(stage + pix * OS + c8);
            if (oy < Ho && ox < Wo)
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + (((int64_t)at.n * Ho + oy) * Wo + ox) * CO + c8));
        }
        if (tile + 1 < last) __syncthreads();   // the staged tile is read before the next patch lands on it
    }
}

// ------------------------------------------------------------------------------- weight gradient
// LDS: the two tiles, and at the end the accumulators of the waves that share a channel-block pair.
constexpr int WG_RS = 36;   // floats per row of a staged 32 x 32 accumulator block
constexpr int wgrad_lds_for(int ci, int co)
{
    const int tiles = (PH * PW * (ci + 8) + TH * TW * (co + 8)) * 2;
    const int pairs = (ci / 32) * (co / 32);
    const int sums = pairs < 4 ? pairs * 9 * 32 * WG_RS * 4 : 0;
    return tiles > sums ? tiles : sums;
}

// partial[b][o][t][i] = sum over the pixels of workgroup b's tiles of dy[pixel][o] * x[pixel + t][i];
// x [N][Hi][Wi][CI], dy [N][Ho][Wo][CO].  A wave owns one (o block, i block) pair with all nine taps
// (144 accumulator registers) and, when there are fewer than four pairs, a share of the tile's rows.
// Per 16 pixels of a tile row it reads the three patch rows under them once, 18 pixels wide, and
// forms the fragments of the three horizontal taps by shifting registers; going down the tile, two
// of the three rows are kept from the step before.  The accumulators leave room for one workgroup
// per CU, so two tiles are on their way into registers meanwhile: one does not cover the memory latency.
template <int CI, int CO>
__global__ __launch_bounds__(NTHREADS) void conv3x3_wgrad_direct_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                                        float* __restrict__ partial, int Hi, int Wi, int Ho, int Wo,
                                                                        int pad, int tiles_x, int tiles_y, int ntiles, int tiles_per_wg)
{
    typedef Rect<PH, PW, CI> Patch;
    typedef Rect<TH, TW, CO> Grad;
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    constexpr int PS = Patch::LD, OS = Grad::LD;
    constexpr int NBI = CI / 32, NBLK = NBI * (CO / 32);   // 1, 2 or 4 channel-block pairs
    constexpr int NP = 4 / NBLK;                            // waves per pair, each with TH / NP tile rows
    constexpr int ROWS = TH / NP;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* patch = reinterpret_cast<bf16_t*>(smem);
    bf16_t* grad = patch + PH * PW * PS;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pair = wave % NBLK, part = wave / NBLK;
    const int jo = pair / NBI, ji = pair % NBI;
    const int row0 = part * ROWS;
    const int first = blockIdx.x * tiles_per_wg, last = min(first + tiles_per_wg, ntiles);

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

    // Pixels p .. p + 9 (p = 8 * (lane >> 5) within the 16-pixel step) of channel 32 ji + (lane & 31)
    // as five dwords: three transposing reads, addressed as in km_frag.
    const int blk = lane >> 4, s4 = lane & 15;
    const int tr_off = (8 * (blk >> 1) + (s4 >> 2)) * PS + ji * 32 + 16 * (blk & 1) + 4 * (s4 & 3);
    struct Row { uint32_t d0, d1, d2, d3, d4; };   // (named fields, not an array: an array ends up in scratch memory)
    auto read_row = [&](int prow, int c) {
        const bf16_t* p = patch + (prow * PW + 16 * c) * PS + tr_off;
        const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
        const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 4 * PS));
        const s16x4 e = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 8 * PS));
        const u32x2 a2 = __builtin_bit_cast(u32x2, a), b2 = __builtin_bit_cast(u32x2, b), e2 = __builtin_bit_cast(u32x2, e);
        return Row{a2.x, a2.y, b2.x, b2.y, e2.x};
    };
    // the 8 pixels starting v pixels to the right
    auto shift0 = [](Row r) { return __builtin_bit_cast(bf16x8, u32x4{r.d0, r.d1, r.d2, r.d3}); };
    auto shift1 = [](Row r) {
        return __builtin_bit_cast(bf16x8, u32x4{__builtin_amdgcn_alignbyte(r.d1, r.d0, 2), __builtin_amdgcn_alignbyte(r.d2, r.d1, 2),
                                                __builtin_amdgcn_alignbyte(r.d3, r.d2, 2), __builtin_amdgcn_alignbyte(r.d4, r.d3, 2)});
    };
    auto shift2 = [](Row r) { return __builtin_bit_cast(bf16x8, u32x4{r.d1, r.d2, r.d3, r.d4}); };

    Patch nx0, nx1;
    Grad nd0, nd1;
    auto fetch = [&](int tile, Patch& nx, Grad& nd) {
        const TileAt at = tile_at(tile, tiles_x, tiles_y);
        nx.fetch(x + (int64_t)at.n * Hi * Wi * CI, Hi, Wi, at.y0 - pad, at.x0 - pad, tid);
        nd.fetch(dy + (int64_t)at.n * Ho * Wo * CO, Ho, Wo, at.y0, at.x0, tid);
    };
    auto step = [&](int tile, Patch& nx, Grad& nd) {
        nx.to_lds(patch, tid);
        nd.to_lds(grad, tid);
        __syncthreads();
        if (tile + 2 < last) fetch(tile + 2, nx, nd);
        // (rolled loops: unrolled, the scheduler hoists the reads of the whole tile and runs out of registers)
#pragma unroll 1
        for (int c = 0; c < TW / 16; ++c) {
            Row top = read_row(row0, c), mid = read_row(row0 + 1, c), bot = read_row(row0 + 2, c);
            bf16x8 df = km_frag<OS>(grad + (row0 * TW + 16 * c) * OS, jo, 0, lane);
#pragma unroll 1
            for (int r = 0; r < ROWS; ++r) {
                // the next step's reads are under way while this one is multiplied
                Row below = bot;
                bf16x8 dfn = df;
                if (r + 1 < ROWS) {
                    below = read_row(row0 + r + 3, c);
                    dfn = km_frag<OS>(grad + ((row0 + r + 1) * TW + 16 * c) * OS, jo, 0, lane);
                }
                // rows <-> i (values), columns <-> o (lane)
                acc[0] = mfma32(shift0(top), df, acc[0]);
                acc[1] = mfma32(shift1(top), df, acc[1]);
                acc[2] = mfma32(shift2(top), df, acc[2]);
                acc[3] = mfma32(shift0(mid), df, acc[3]);
                acc[4] = mfma32(shift1(mid), df, acc[4]);
                acc[5] = mfma32(shift2(mid), df, acc[5]);
                acc[6] = mfma32(shift0(bot), df, acc[6]);
                acc[7] = mfma32(shift1(bot), df, acc[7]);
                acc[8] = mfma32(shift2(bot), df, acc[8]);
                top = mid;
                mid = bot;
                bot = below;
                df = dfn;
            }
        }
        if (tile + 1 < last) __syncthreads();   // all fragments are read before the next tile lands
    };
    fetch(first, nx0, nd0);
    if (first + 1 < last) fetch(first + 1, nx1, nd1);
    for (int tile = first; tile < last; tile += 2) {
        step(tile, nx0, nd0);
        if (tile + 1 < last) step(tile + 1, nx1, nd1);
    }

    // The waves of a pair add up in a fixed order through LDS; the last one writes the partial.
    // lane holds, for o = 32 jo + (lane & 31), the input channels 32 ji + 8 g + 4 h + 0..3
    const int h = lane >> 5;
    if (NP > 1) {
        float* sums = reinterpret_cast<float*>(smem) + (pair * 9 * 32 + (lane & 31)) * WG_RS + 4 * h;
        __syncthreads();   // the tiles are not needed any more
#pragma unroll
        for (int p = 0; p + 1 < NP; ++p) {
            if (part == p) {
#pragma unroll
                for (int t = 0; t < 9; ++t)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        f32x4 v = {acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
                        f32x4* at = reinterpret_cast<f32x4*>(sums + t * 32 * WG_RS + 8 * g);
                        if (p > 0) v += *at;
                        *at = v;
                    }
            }
            __syncthreads();
        }
        if (part != NP - 1) return;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(sums + t * 32 * WG_RS + 8 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[t][4 * g + e] += v[e];
            }
    }
    float* dst = partial + (((int64_t)blockIdx.x * CO + jo * 32 + (lane & 31)) * 9) * CI + ji * 32 + 4 * h;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 v = {acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
            *reinterpret_cast<f32x4*>(dst + t * CI + 8 * g) = v;
        }
}

// --------------------------------------------------------------------------------------- host side
struct Tiling { int tiles_x, tiles_y; int64_t ntiles; };
inline Tiling tiling(int N, int Ho, int Wo)
{
    Tiling t;
    t.tiles_x = (int)ceil_div(Wo, TW);
    t.tiles_y = (int)ceil_div(Ho, TH);
    t.ntiles = (int64_t)N * t.tiles_x * t.tiles_y;
    return t;
}

template <class K>
hipError_t allow_lds(K kern, int lds, bool* done)
{
    if (*done) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    *done = e == hipSuccess;
    return e;
}

template <int CI, int CO, bool WT>
hipError_t launch_conv(const bf16_t* in, const bf16_t* w, bf16_t* out, int N, int Hi, int Wi, int Ho, int Wo, int pad, hipStream_t st)
{
    constexpr int lds = conv_lds_bytes<CI, CO, WT>();
    auto kern = conv3x3_direct_kernel<CI, CO, WT>;
    static bool allowed = false;
    hipError_t e = allow_lds(kern, lds, &allowed);
    if (e != hipSuccess) return e;
    const Tiling t = tiling(N, Ho, Wo);
    // about as many workgroups as fit on the chip at once (LDS decides), each with a run of tiles
    const int resident = 256 * std::max(1, (160 * 1024) / lds);
    const int tiles_per_wg = (int)std::min<int64_t>(std::max<int64_t>(t.ntiles / resident, 1), 8);
    hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div(t.ntiles, tiles_per_wg)), dim3(NTHREADS), lds, st, in, w, out, Hi, Wi, Ho, Wo, pad,
                       t.tiles_x, t.tiles_y, (int)t.ntiles, tiles_per_wg);
    return hipGetLastError();
}

// Workgroups (= partial slices) of the weight gradient: one per CU, fewer when there are fewer tiles.
inline int wgrad_tiles_per_wg(int64_t ntiles) { return (int)std::max<int64_t>(ceil_div(ntiles, 256), 1); }

template <int CI, int CO>
hipError_t launch_wgrad(const bf16_t* x, const bf16_t* dy, float* partial, int N, int Hi, int Wi, int Ho, int Wo, int pad, int* slices,
                        hipStream_t st)
{
    constexpr int lds = wgrad_lds_for(CI, CO);
    auto kern = conv3x3_wgrad_direct_kernel<CI, CO>;
    static bool allowed = false;
    hipError_t e = allow_lds(kern, lds, &allowed);
    if (e != hipSuccess) return e;
    const Tiling t = tiling(N, Ho, Wo);
    const int tiles_per_wg = wgrad_tiles_per_wg(t.ntiles);
    *slices = (int)ceil_div(t.ntiles, tiles_per_wg);
    hipLaunchKernelGGL(kern, dim3((unsigned)*slices), dim3(NTHREADS), lds, st, x, dy, partial, Hi, Wi, Ho, Wo, pad, t.tiles_x, t.tiles_y,
                       (int)t.ntiles, tiles_per_wg);
    return hipGetLastError();
}

inline bool small(int c) { return c == 32 || c == 64; }

inline bool shape_ok(const ConvShape& cs)
{
    if (cs.k != 3 || cs.stride != 1 || cs.pad < 0 || cs.pad > 2 || !small(cs.I) || !small(cs.O)) return false;
    if (cs.N < 1 || cs.Ho < 1 || cs.Wo < 1 || cs.Ho != cs.H + 2 * cs.pad - 2 || cs.Wo != cs.W + 2 * cs.pad - 2) return false;
    // tile counts and pixel offsets stay in 32 bits
    return (int64_t)cs.N * ceil_div(cs.H + 2, TH) * ceil_div(cs.W + 2, TW) < (int64_t(1) << 31) &&
           (int64_t)(cs.H + 2) * (cs.W + 2) * 64 < (int64_t(1) << 31);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

size_t conv_direct_wgrad_bytes(const ConvShape& cs, bool bf16)
{
    if (!bf16 || !shape_ok(cs)) return 0;
    const Tiling t = tiling(cs.N, cs.Ho, cs.Wo);
    const int64_t slices = ceil_div(t.ntiles, wgrad_tiles_per_wg(t.ntiles));
    return (size_t)slices * 9 * cs.I * cs.O * sizeof(float);
}

bool conv_direct_supported(const MatOp& op)
{
    if (op.gather == GATHER_NONE || !op.in_bf16 || op.bias || op.epilogue != EPI_NONE || !shape_ok(op.cs)) return false;
    if (!aligned16(op.A) || !aligned16(op.B) || !aligned16(op.C)) return false;
    const ConvShape& cs = op.cs;
    switch (op.gather) {
    case GATHER_CONV_FWD:     // A = x [pixels][I], B = w [O][9 I], C = y [pixels][O]
        return !op.out_f32 && op.splits <= 1 && op.a_sm == cs.I && op.a_sk == 1 && op.b_sn == 9 * cs.I && op.b_sk == 1 &&
               op.ldc == cs.O;
    case GATHER_CONV_DGRAD:   // A = dy [pixels][O], B = w, C = dx [pixels][I]
        return !op.out_f32 && op.splits <= 1 && op.a_sm == cs.O && op.a_sk == 1 && op.ldc == cs.I;
    case GATHER_CONV_WGRAD:   // A = dy read as [O][pixels], B = x read as [9 I][pixels], C = dw [O][9 I] fp32
        return op.out_f32 && op.a_sm == 1 && op.a_sk == cs.O && op.b_sn == 1 && op.b_sk == cs.I && op.ldc == 9 * cs.I &&
               op.scratch && aligned16(op.scratch) && op.scratch_bytes >= conv_direct_wgrad_bytes(cs, true);
    }
    return false;
}

hipError_t conv_direct(const MatOp& op, hipStream_t st)
{
    note_kernel("conv3x3_direct (patch staging)");
    const ConvShape& cs = op.cs;
    const bf16_t* A = (const bf16_t*)op.A;
    const bf16_t* B = (const bf16_t*)op.B;
    const int ci = op.gather == GATHER_CONV_DGRAD ? cs.O : cs.I, co = op.gather == GATHER_CONV_DGRAD ? cs.I : cs.O;
    const int sel = (ci == 64 ? 2 : 0) + (co == 64 ? 1 : 0);
    if (op.gather == GATHER_CONV_FWD) {
        bf16_t* y = (bf16_t*)op.C;
        switch (sel) {
        case 0: return launch_conv<32, 32, false>(A, B, y, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, st);
        case 1: return launch_conv<32, 64, false>(A, B, y, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, st);
        case 2: return launch_conv<64, 32, false>(A, B, y, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, st);
        default: return launch_conv<64, 64, false>(A, B, y, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, st);
        }
    }
    if (op.gather == GATHER_CONV_DGRAD) {
        // dx [N][H][W][I] = convolution of dy [N][Ho][Wo][O] with padding 2 - pad
        bf16_t* dx = (bf16_t*)op.C;
        switch (sel) {
        case 0: return launch_conv<32, 32, true>(A, B, dx, cs.N, cs.Ho, cs.Wo, cs.H, cs.W, 2 - cs.pad, st);
        case 1: return launch_conv<32, 64, true>(A, B, dx, cs.N, cs.Ho, cs.Wo, cs.H, cs.W, 2 - cs.pad, st);
        case 2: return launch_conv<64, 32, true>(A, B, dx, cs.N, cs.Ho, cs.Wo, cs.H, cs.W, 2 - cs.pad, st);
        default: return launch_conv<64, 64, true>(A, B, dx, cs.N, cs.Ho, cs.Wo, cs.H, cs.W, 2 - cs.pad, st);
        }
    }
    float* partial = (float*)op.scratch;
    int slices = 0;
    hipError_t e;
    switch (sel) {   // A = dy, B = x
    case 0: e = launch_wgrad<32, 32>(B, A, partial, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, &slices, st); break;
    case 1: e = launch_wgrad<32, 64>(B, A, partial, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, &slices, st); break;
    case 2: e = launch_wgrad<64, 32>(B, A, partial, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, &slices, st); break;
    default: e = launch_wgrad<64, 64>(B, A, partial, cs.N, cs.H, cs.W, cs.Ho, cs.Wo, cs.pad, &slices, st); break;
    }
    if (e != hipSuccess) return e;
    return reduce_partials(partial, op.C, false, op.ldc, cs.O, 9 * (int64_t)cs.I, slices, st, op.sgd);
}

}  // namespace lrd
