// ReuseCert (Appendix C, "ReuseCert"; Section 6.1) through a layer that sits above a convolutional front: the replacement step
//     stored_k = [W+ | W- | b] x [Lr ; Ur ; unit row]          (lower side; the upper side swaps W+ and W-)
// as an implicit contraction, fp32 MFMA (v_mfma_f32_32x32x2_f32), without writing the gathered operand out.
//
// The stored input-level bounds of a convolution neuron reach only its receptive field, so a row of Rr holds a window of
// ph_i x pw_i x C0 input positions (corner of neuron (y, x) at (y*S_i - P_i, x*S_i - P_i)) and the constant behind it.  The
// layer on top -- a convolution, or a fully-connected layer read as a convolution whose kernel covers the whole grid -- adds
// the rows of the neurons it reads, each placed at its own offset inside the output frame (the window of the output position,
// or the whole image).  Per output position z, tap t = (ky, kx) and channel ci the contraction therefore multiplies
//     A[m][part, t, ci]  (split weights of output neuron m; part 0 multiplies Lr, part 1 Ur)
// with row (part, neuron(t), ci) of Rr[input of z], shifted: frame column (qy, qx, c) reads window column
// (qy - oy_t, qx - ox_t, c) of that row, or nothing when that falls outside the window.
//
// Work split: a workgroup (4 wavefronts) owns 32*MT rows m (both sides stacked: m < M is the lower side, the rest the upper
// side) x four 32-column blocks of the frame of one output position, one block per wavefront for all the rows.  Where a frame
// row fills its 32-column blocks (at least 9 lanes of 10), the four blocks are the same block of four consecutive frame
// rows: a tap's window covers the same columns in every row, so the wavefronts meet the same taps and finish together, and
// taps that miss the tile in either direction are skipped by the whole workgroup; the constant column is then one more
// frame row.  Narrow frames take 128 consecutive columns of the flattened frame instead (taps are skipped by frame rows for
// the workgroup and by block for a wavefront).  The A operand of one (tap, chunk of 32 channels) goes through LDS,
// k-contiguous per row so that four reduction steps come from one 16-byte read (row stride 2*CK + 4 floats: conflict-free);
// the B operand comes straight from global memory (L2), one float per lane per step through a buffer resource whose
// out-of-range offsets read zeros (so a lane outside the window needs no branch), fetched eight steps ahead.  One MFMA step
// consumes Lr row ci (lanes 0-31, k = 0) and Ur row ci (lanes 32-63, k = 1).
// Summation order is fixed (taps in order, channels in order), so results are reproducible.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "conv.h"

namespace dpc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float vf4 __attribute__((ext_vector_type(4)));

constexpr int kRwThreads = 256;

struct RwArgs {
    const float* A0; const float* A1;   // split weights of the lower / upper side [M][ld_split]
    int ld_split, kk, M, Ci;            // kk = taps * Ci: column of part 1; column 2*kk holds the bias
    const float* Rr;                    // [batch][2*n + 1][ld_i]
    long long rr_block;                 // floats per input: (2*n + 1) * ld_i
    int n, ld_i;
    int ph_i, pw_i, C0, S_i, P_i;       // windows of the rows of Rr
    int kh, kw, stride, pad, H, W, Wo, npos;   // taps of the layer, grid it reads (H x W x Ci), its output positions
    int fh, fw, ld_o, S_o, P_o, frame_image;   // output frame: window of the output position (origin ho*S_o - P_o), or the image
    float* E;                           // [side][batch * npos * M][ld_o]
    long long side_stride;              // floats between the two sides of E
    int CK;                             // channels per staged chunk (divides Ci, multiple of 8)
    int n_xt;                           // 32-float blocks per frame row
    int flat;                           // tiles over the flattened frame instead of over frame rows
    int gx, gy;                         // column tiles and row blocks per output position
    long long total;                    // workgroups with work: gx * gy * output positions
};

template <int MT>
__global__ __launch_bounds__(kRwThreads, 2) void reuse_window_kernel(RwArgs a)
{
    extern __shared__ float4 lds4[];
    float* sA = reinterpret_cast<float*>(lds4);                    // [32*MT][2*CK + 4]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kq = lane >> 5;
    // Workgroup -> (row block, column tile, output position), row block fastest.  Workgroups are dealt to the 8 XCDs round
    // robin, so consecutive indices ON ONE XCD (blockIdx.x = xcd + 8 * slot) take consecutive work items: the row blocks of one
    // tile, then the neighbouring tiles and positions, which read the same rows of Rr, share that XCD's L2.
    const long long per = (a.total + 7) >> 3;
    const long long item = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
    if (item >= a.total) return;
    const int by = (int)(item % a.gy);
    const long long rest = item / a.gy;
    const int bx = (int)(rest % a.gx);
    const long long z = rest / a.gx;
    const int b = (int)(z / a.npos), pos = (int)(z - (long long)b * a.npos);
    const int ho = pos / a.Wo, wo = pos - ho * a.Wo;
    const int elems_o = a.fh * a.fw * a.C0, elems_i = a.ph_i * a.pw_i * a.C0;
    const int astride = 2 * a.CK + 4;
    const int mbase = by * 32 * MT;

    // The workgroup's tile, one 32-column block per wavefront.
    // Row tiles: block xt of four consecutive frame rows, so the four wavefronts meet the same taps (a tap's window covers
    // the same columns in every row) and finish together; the constant column counts as one more frame row with a single
    // column, the rest of that row's block being the padding of the stored row.
    // Flat tiles (frames whose rows would leave many lanes of a 32-column block empty): 128 consecutive columns of the
    // flattened frame, constant and padding included; the wavefronts then differ in the taps they can skip.
    const int rowlen = a.fw * a.C0;
    int qy, qx, qc, ncol, ty_lo, ty_hi, tx_lo, tx_hi;
    bool is_const, in_frame, wg_const, stores;
    if (a.flat) {
        const int col0 = bx * 128;
        ncol = col0 + wave * 32 + l32;
        is_const = ncol == elems_o;
        in_frame = ncol < elems_o;
        const int q = ncol / a.C0;
        qc = ncol - q * a.C0;
        qy = q / a.fw;
        qx = q - qy * a.fw;
        wg_const = col0 <= elems_o && elems_o < col0 + 128;
        ty_lo = col0 / rowlen;
        ty_hi = col0 < elems_o ? (std::min(col0 + 128, elems_o) - 1) / rowlen : -1;
        tx_lo = 0;
        tx_hi = rowlen - 1;
        stores = ncol < a.ld_o;
    } else {
        const int xt = bx % a.n_xt, rg = bx / a.n_xt;
        const int xcol = xt * 32 + l32;
        qy = rg * 4 + wave;                                        // frame row of this wavefront (fh: the constant's row)
        const bool const_row = qy == a.fh;
        is_const = const_row && xcol == 0;
        in_frame = qy < a.fh && xcol < rowlen;
        qx = xcol / a.C0;
        qc = xcol - qx * a.C0;
        wg_const = rg * 4 <= a.fh && a.fh < rg * 4 + 4 && xt == 0;
        ty_lo = rg * 4;
        ty_hi = std::min(rg * 4 + 3, a.fh - 1);
        tx_lo = xt * 32;
        tx_hi = std::min(xt * 32 + 31, rowlen - 1);
        ncol = const_row ? elems_o + l32 : qy * rowlen + xcol;
        stores = in_frame || (const_row && xt == 0 && ncol < a.ld_o);
    }
    const int fy0 = a.frame_image ? 0 : ho * a.S_o - a.P_o, fx0 = a.frame_image ? 0 : wo * a.S_o - a.P_o;

    constexpr int kOutside = (int)0x80000000;
    const __amdgpu_buffer_rsrc_t bres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.Rr + (size_t)b * a.rr_block), 0, (int)(a.rr_block * 4), 0x00020000);
    const int part_off = kq * a.n * a.ld_i * 4;                    // bytes from an Lr row to the Ur row of the same neuron

    floatx16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mt][v] = 0.0f;

    for (int ky = 0; ky < a.kh; ++ky) {
        const int y = ho * a.stride - a.pad + ky;
        if (y < 0 || y >= a.H) continue;                           // zero padding: no neuron
        const int oy = y * a.S_i - a.P_i - fy0;                    // frame row of the window's first row
        if (!wg_const && (ty_hi < ty_lo || oy > ty_hi || oy + a.ph_i <= ty_lo)) continue;
        const int py = qy - oy;
        const bool row_ok = py >= 0 && py < a.ph_i;
        for (int kx = 0; kx < a.kw; ++kx) {
            const int x = wo * a.stride - a.pad + kx;
            if (x < 0 || x >= a.W) continue;
            const int ox = x * a.S_i - a.P_i - fx0;
            if (!wg_const && (tx_hi < tx_lo || ox * a.C0 > tx_hi || (ox + a.pw_i) * a.C0 <= tx_lo)) continue;
            const int t = ky * a.kw + kx;
            const int nrow0 = (y * a.W + x) * a.Ci;                // first of the neuron rows of this tap
            const int px = qx - ox;
            const bool valid = in_frame && row_ok && px >= 0 && px < a.pw_i;
            const int voff = valid ? ((py * a.pw_i + px) * a.C0 + qc) * 4 + part_off : is_const ? elems_i * 4 + part_off : kOutside;
            const bool wave_live = __ballot(valid || is_const) != 0ull;
            for (int c0 = 0; c0 < a.Ci; c0 += a.CK) {
                float bcur[8], bnxt[8];
                auto load_b = [&](float (&bb)[8], int s0) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        bb[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(bres, voff, (nrow0 + c0 + s0 + u) * a.ld_i * 4, 0));
                };
                if (wave_live) load_b(bcur, 0);                    // in flight while the A chunk is staged
                __syncthreads();                                   // every wavefront is done with the previous chunk
                {
                    // several 16-byte loads in flight per thread before the first LDS write
                    constexpr int kU = 4;
                    const int q4n = a.CK >> 1;                     // 16-byte pieces per row: 2 parts x CK / 4
                    const int total = 32 * MT * q4n;
                    for (int idx0 = tid; idx0 < total; idx0 += kRwThreads * kU) {
                        vf4 v[kU];
                        int dsto[kU];
#pragma unroll
                        for (int u = 0; u < kU; ++u) {
                            const int idx = idx0 + u * kRwThreads;
                            const int row = idx / q4n, q4 = idx - row * q4n;
                            const int part = q4 >= (a.CK >> 2), c4 = q4 - part * (a.CK >> 2);
                            const int m = mbase + row;
                            const int side = m >= a.M, r = m - side * a.M;
                            v[u] = vf4{0.f, 0.f, 0.f, 0.f};
                            if (idx < total && m < 2 * a.M)
                                v[u] = *reinterpret_cast<const vf4*>((side ? a.A1 : a.A0) + (size_t)r * a.ld_split + part * a.kk + t * a.Ci + c0 + c4 * 4);
                            dsto[u] = idx < total ? row * astride + part * a.CK + c4 * 4 : -1;
                        }
#pragma unroll
                        for (int u = 0; u < kU; ++u)
                            if (dsto[u] >= 0) *reinterpret_cast<vf4*>(sA + dsto[u]) = v[u];
                    }
                }
                __syncthreads();
                if (!wave_live) continue;
                const float* arow = sA + l32 * astride + kq * a.CK;
                for (int s0 = 0; s0 < a.CK; s0 += 8) {
                    if (s0 + 8 < a.CK) load_b(bnxt, s0 + 8);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        vf4 av[MT];
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) av[mt] = *reinterpret_cast<const vf4*>(arow + mt * 32 * astride + s0 + 4 * h);
#pragma unroll
                        for (int u = 0; u < 4; ++u)
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mt][u], bcur[4 * h + u], acc[mt], 0, 0, 0);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) bcur[u] = bnxt[u];
                }
            }
        }
    }

    // ---- epilogue: accumulator register 4*i + j of a lane is row 8*i + 4*kq + j, column l32 ----
    // (lanes on the padding of the stored rows hold zeros)
    if (!stores) return;
    float* Eb = a.E + ((size_t)z * a.M) * a.ld_o + ncol;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = mbase + mt * 32 + 8 * i + 4 * kq + j;
                if (m >= 2 * a.M) continue;
                const int side = m >= a.M, r = m - side * a.M;
                float v = acc[mt][4 * i + j];
                if (is_const) v += (side ? a.A1 : a.A0)[(size_t)r * a.ld_split + 2 * a.kk];      // the unit row carries the bias
                Eb[(size_t)side * a.side_stride + (size_t)r * a.ld_o] = v;
            }
}

}  // namespace



bool reuse_window_covers(int Ci) { return Ci >= 8 && Ci % 8 == 0; }

double launch_reuse_window(const float* A0, const float* A1, int ld_split, int M, const float* Rr, int n, const ReuseWindow& fi, const ConvGeom& g,
                           int fh, int fw, int ld_o, int S_o, int P_o, bool frame_image, int batch, float* E, hipStream_t s)
{
    const int kk = g.kh * g.kw * g.Ci;
    const int64_t npos = (int64_t)g.Ho * g.Wo, nz = (int64_t)batch * npos;
    const int64_t rr_block = (2 * (int64_t)n + 1) * fi.ld;
    DPC_REQUIRE(A0 && A1 && Rr && E && M >= 1 && batch >= 0 && reuse_window_covers(g.Ci) && n == g.Ci * g.H * g.W, DPC_EINVAL,
                "reuse_window: bad arguments");
    DPC_REQUIRE(ld_split > 2 * kk && ld_split % 4 == 0 && fi.ld > fi.ph * fi.pw * fi.C0 && ld_o > fh * fw * fi.C0 && fi.C0 >= 1 &&
                    ((uintptr_t)A0 % 16) == 0 && ((uintptr_t)A1 % 16) == 0, DPC_EINVAL, "reuse_window: bad layout");
    DPC_REQUIRE(rr_block * 4 < ((int64_t)1 << 31) && nz * M < ((int64_t)1 << 31), DPC_EINVAL, "reuse_window: operand too large");
    if (nz == 0) return 0.0;
    RwArgs a{};
    a.A0 = A0; a.A1 = A1; a.ld_split = ld_split; a.kk = kk; a.M = M; a.Ci = g.Ci;
    a.Rr = Rr; a.rr_block = rr_block; a.n = n; a.ld_i = fi.ld;
    a.ph_i = fi.ph; a.pw_i = fi.pw; a.C0 = fi.C0; a.S_i = fi.S; a.P_i = fi.P;
    a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pad = g.pad; a.H = g.H; a.W = g.W; a.Wo = g.Wo; a.npos = (int)npos;
    a.fh = fh; a.fw = fw; a.ld_o = ld_o; a.S_o = S_o; a.P_o = P_o; a.frame_image = frame_image ? 1 : 0;
    a.E = E; a.side_stride = nz * M * ld_o;
    const int g_rw_ck = tune(TK_REUSE_WINDOW_CK), g_rw_flat = tune(TK_REUSE_WINDOW_TILES);   // 0 / -1: by shape
    a.CK = (g_rw_ck >= 8 && g_rw_ck <= 64 && g_rw_ck % 8 == 0 && g.Ci % g_rw_ck == 0) ? g_rw_ck : g.Ci <= 32 ? g.Ci : g.Ci % 32 == 0 ? 32 : g.Ci % 16 == 0 ? 16 : 8;
    const int rows = 2 * M;
    const int MT = rows > 64 ? 4 : rows > 32 ? 2 : 1;
    a.n_xt = ceil_div(fw * fi.C0, 32);
    const int n_rg = fh / 4 + 1;                                  // row groups: the constant's row fh is one of the rows
    // row tiles when at least 9 of 10 lanes of a row's blocks hold a column
    a.flat = g_rw_flat >= 0 ? g_rw_flat : (fw * fi.C0 * 10 < a.n_xt * 32 * 9);
    const size_t lds = (size_t)32 * MT * (2 * a.CK + 4) * 4;
    const unsigned gx = a.flat ? (unsigned)ceil_div(ld_o, 128) : (unsigned)(a.n_xt * n_rg), gy = (unsigned)ceil_div(rows, 32 * MT);
    constexpr int kMaxLds = 32 * 4 * (2 * 64 + 4) * 4;
    auto go = [&](auto kern, const dim3& grid) {
        ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kMaxLds);
        hipLaunchKernelGGL(kern, grid, dim3(kRwThreads), lds, s, a);
    };
    a.gx = (int)gx;
    a.gy = (int)gy;
    a.total = (int64_t)gx * gy * nz;
    DPC_REQUIRE(a.total + 8 < ((int64_t)1 << 31), DPC_EINVAL, "reuse_window: too many workgroups");
    const dim3 grid((unsigned)(ceil_div(a.total, 8) * 8));
    if (MT == 4) go(&reuse_window_kernel<4>, grid);
    else if (MT == 2) go(&reuse_window_kernel<2>, grid);
    else go(&reuse_window_kernel<1>, grid);
    DPC_HIP(hipGetLastError());
    // multiply-adds of the taps that exist, over whole windows (what the step computes; skipped lanes do not count)
    double taps = 0.0;
    for (int ho = 0; ho < g.Ho; ++ho)
        for (int ky = 0; ky < g.kh; ++ky) {
            const int y = ho * g.stride - g.pad + ky;
            if (y < 0 || y >= g.H) continue;
            for (int wo = 0; wo < g.Wo; ++wo)
                for (int kx = 0; kx < g.kw; ++kx) {
                    const int x = wo * g.stride - g.pad + kx;
                    if (x >= 0 && x < g.W) taps += 1.0;
                }
        }
    return 2.0 * 2.0 * (double)batch * taps * M * (2.0 * g.Ci) * (fi.ph * fi.pw * fi.C0 + 1);
}

}  // namespace dpc
