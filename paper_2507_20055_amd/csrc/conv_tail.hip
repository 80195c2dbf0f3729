// Tail of a traversal of convolution-layer rows (Patches form) in one kernel: the last ReLU step, the transposed
// convolution through the network's first layer (few input channels: the image) and the concretisation against
// the box, without the coefficients touching HBM again:
//
//   in rows (patch over the first ReLU layer)  --sign-split ReLU step-->  A operand of the MFMA product with all
//   taps  -->  P panel in LDS  --ordered gather-->  coefficients over the image (registers)  --box-->  one bound.
//
// Replaces three launches (ReLU step: read + write of the rows; product-then-gather convolution: read, write of
// the image-level rows; concretisation: read).  The arithmetic of each stage is that of the separate kernels:
// x' = x * mult, c += x * k with (mult, k) chosen by the sign of x and the side of the row; the per-position product
// P[(row, position)][(tap, ci)] = sum_co x' * K; every output coefficient gathers its taps in a fixed order; the
// bound adds coefficient * (lo or hi by sign and side) over the positions that lie on the image.
//
// A workgroup takes RB consecutive rows; RB divides the number of output channels of the bounded layer, so the
// rows of a panel belong to one (side, input) group and one spatial position of that layer: they share the patch
// origin, i.e. the same window of ReLU parameters and of the box.
#include <algorithm>
#include <type_traits>

#include "conv.h"

namespace dpc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float vf4 __attribute__((ext_vector_type(4)));

constexpr int kTailThreads = 256;

struct TailArgs {
    const float* in; int ld_in;                    // rows [M][ld_in]; SHARED: cores [rows_C][ld_in]
    const double* cst; const float* cst_init_c;    // row constants [M]; SHARED: per-core constants [rows_C]
    long long M; int R, batch, rows_W, rows_C;
    int ih, iw;                                    // patch extent over the ReLU layer (CO channels)
    int pS, pP, gh, gw;                            // patch origin = index * pS - pP on the ReLU layer's grid gh x gw
    const float2* pk2; int ldpk; const float* bias_c;   // (mu, nu | lambda in the sign) [batch][ldpk]; conv bias per channel
    const float* taps; int Ci, kh, kw;             // first layer's kernel [kh][kw][CO][Ci]
    int oh, ow;                                    // output patch extent
    int qS, qP, H, W;                              // output patch origin = index * qS - qP on the image H x W x Ci
    const float* lo; const float* hi;              // box [batch][H*W*Ci]
    float* out_l; float* out_u;                    // [batch][R]
    int RB, panels;
};

template <int NT, int S, int CO8, bool SHARED>
__global__ __launch_bounds__(kTailThreads, 2) void patch_tail_kernel(TailArgs a)
{
    constexpr int CO = CO8 * 8, NC = 32 * NT, PS = NC + 3, NW = kTailThreads / 64;
    extern __shared__ float4 lds4[];
    const int npos = a.ih * a.iw, E = a.RB * npos, ntiles = (E + 31) >> 5, E32 = ntiles * 32;
    const int Pout = a.oh * a.ow;
    float* sP = reinterpret_cast<float*>(lds4);        // [E32][PS]
    const int zoff = E32 * PS;                         // four zeros
    float* sK = sP + zoff + 4;                         // [E32] row-constant contribution of every entry
    float* sC = sK + E32;                              // [RB * Pout] bound contribution of every output position
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kq = lane >> 5;
    const int CI = a.Ci;
    const int ncols = a.kh * a.kw * CI;
    const unsigned long long magic_pout = (1ull << 32) / (unsigned)max(Pout, 1) + 1;
    const unsigned long long magic_ow = (1ull << 32) / (unsigned)max(a.ow, 1) + 1;
    if (tid < 4) sP[zoff + tid] = 0.0f;

    // kernel matrix in the B-operand layout: step (g, s4) of the reduction multiplies channel 8g + 4kq + s4
    float bk[NT][CO8 * 4];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int col = n * 32 + l32;
        const int tap = col / CI, ci = col - tap * CI;
#pragma unroll
        for (int k = 0; k < CO8 * 4; ++k) {
            const int co = 8 * (k >> 2) + 4 * kq + (k & 3);
            bk[n][k] = col < ncols ? a.taps[((size_t)tap * CO + co) * CI + ci] : 0.0f;
        }
    }
    float bias[CO8][4];                                // conv bias of this lane's channels
#pragma unroll
    for (int g = 0; g < CO8; ++g)
#pragma unroll
        for (int k = 0; k < 4; ++k) bias[g][k] = a.bias_c[8 * g + 4 * kq + k];

    // Tiles are fetched (rows and ReLU parameters) one step ahead, across panel boundaries too: the loads of the next
    // step are in flight during the MFMAs of this one and during the gather and reduction phases.  Lanes whose entry
    // lies outside the panel, the row range or the layer's grid hold zeros, which contribute nothing below.
    constexpr int T = 1;                               // tiles per step (two cost registers and with them a wavefront per SIMD)
    const int ipp = (ntiles + T * NW - 1) / (T * NW);                  // steps per wavefront per panel
    const unsigned long long magic_npos = (1ull << 32) / (unsigned)max(npos, 1) + 1;     // e / npos for e * npos < 2^32
    const unsigned long long magic_iw = (1ull << 32) / (unsigned)max(a.iw, 1) + 1;
    // Position of a panel: consecutive panels are RB rows apart, so the decomposition of the first row is carried from
    // panel to panel with a few scalar compares instead of being divided out again (RB divides rows_C, rows_C divides R).
    struct Pos { long long m0; int grp, r0, co0, wo, ho; };
    auto first_pos = [&](long long m0) __attribute__((always_inline)) {
        Pos p;
        p.m0 = m0;
        p.grp = (int)(m0 / a.R);
        p.r0 = (int)(m0 - (long long)p.grp * a.R);
        p.co0 = p.r0 % a.rows_C;
        p.wo = (p.r0 / a.rows_C) % a.rows_W;
        p.ho = p.r0 / (a.rows_C * a.rows_W);
        return p;
    };
    auto advance = [&](Pos p) __attribute__((always_inline)) {
        p.m0 += a.RB; p.r0 += a.RB; p.co0 += a.RB;
        if (p.co0 >= a.rows_C) { p.co0 = 0; if (++p.wo >= a.rows_W) { p.wo = 0; ++p.ho; } }
        if (p.r0 >= a.R) { p.r0 = 0; p.co0 = 0; p.wo = 0; p.ho = 0; ++p.grp; }
        return p;
    };
    auto fetch = [&](const Pos& pp, bool live, int it, vf4 (&X)[T][CO8], float4 (&PK)[T][CO8][2]) __attribute__((always_inline)) {
        const long long m0 = live ? pp.m0 : 0;
        const int grp = live ? pp.grp : 0, co0 = live ? pp.co0 : 0;
        const int b = grp - (grp >= a.batch ? a.batch : 0);
        const int oy = pp.ho * a.pS - a.pP, ox = pp.wo * a.pS - a.pP;  // patch origin on the ReLU layer's grid
        const int t0 = (wave + it * NW) * T;
        // both operands through buffer loads whose resources start at the panel's first row (the bounded layer's cores
        // for shared rows) and at the input's parameter block: 32-bit lane offsets, no branches, no zero fill
        const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(SHARED ? a.in + (size_t)co0 * a.ld_in : a.in + m0 * a.ld_in), 0, live ? a.RB * a.ld_in * 4 : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t qres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float2*>(a.pk2 + (size_t)b * a.ldpk), 0, live ? a.ldpk * 8 : 0, 0x00020000);
        constexpr int kOutside = (int)0x80000000;
#pragma unroll
        for (int u = 0; u < T; ++u) {
            const int e = (t0 + u) * 32 + l32;
            const int ml = (int)(((unsigned long long)e * magic_npos) >> 32), pos = e - ml * npos;
            const int py = (int)(((unsigned long long)pos * magic_iw) >> 32), px = pos - py * a.iw;
            const int gy = oy + py, gx = ox + px;
            const bool ok = live && t0 + u < ntiles && e < E && m0 + ml < a.M && gy >= 0 && gy < a.gh && gx >= 0 && gx < a.gw;
            // a lane outside the panel, the rows or the grid gets an offset outside the resources and reads zeros
            const int xo = ok ? (ml * a.ld_in + pos * CO + 4 * kq) * 4 : kOutside;
            const int qo = ok ? ((gy * a.gw + gx) * CO + 4 * kq) * 8 : kOutside;
#pragma unroll
            for (int g = 0; g < CO8; ++g) {
                X[u][g] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(xres, xo + 32 * g, 0, 0));
                PK[u][g][0] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(qres, qo + 64 * g, 0, 0));
                PK[u][g][1] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(qres, qo + 64 * g + 16, 0, 0));
            }
        }
    };
    vf4 X[T][CO8];
    float4 PK[T][CO8][2];
    Pos cur = first_pos((long long)blockIdx.x * a.panels * a.RB);
    bool cur_live = a.panels > 0 && cur.m0 < a.M;
    fetch(cur, cur_live, 0, X, PK);

    for (int pi = 0; pi < a.panels; ++pi) {
        if (!cur_live) break;                                          // uniform over the workgroup; nothing in flight
        const Pos nxt = advance(cur);
        const bool nxt_live = pi + 1 < a.panels && nxt.m0 < a.M;
        const long long m0 = cur.m0;
        const int r0 = cur.r0, co0 = cur.co0;
        const int side = cur.grp >= a.batch, b = cur.grp - side * a.batch;
        const int qy = cur.ho * a.qS - a.qP, qx = cur.wo * a.qS - a.qP;   // output patch origin on the image

        // ---- ReLU step on the fetched tiles, product with all taps, panel to LDS ----
        for (int it = 0; it < ipp; ++it) {
            const int t0 = (wave + it * NW) * T;
            vf4 av[T][CO8];
            float ks[T];
            // ReLU step, per element x with (mu, nu | lambda) and the bias of its channel: the part of x on which this
            // side takes the upper relaxation is p (x >= 0 on the upper side, x < 0 on the lower side), the rest n:
            //   y = p * mu + lambda * n,   constant += p * (mu * bias + nu) + lambda * n * bias
            auto relu_step = [&](auto upper_side) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < T; ++u) {
                    ks[u] = 0.0f;
#pragma unroll
                    for (int g = 0; g < CO8; ++g) {
                        const vf4 x = X[u][g];
                        const float4 p01 = PK[u][g][0], p23 = PK[u][g][1];
                        const float mu[4] = {p01.x, p01.z, p23.x, p23.z}, nl[4] = {p01.y, p01.w, p23.y, p23.w};
                        vf4 y;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float p = decltype(upper_side)::value ? fmaxf(x[k], 0.0f) : fminf(x[k], 0.0f);
                            const float n = decltype(upper_side)::value ? fminf(x[k], 0.0f) : fmaxf(x[k], 0.0f);
                            // lambda (0 or 1) is the sign bit of the second parameter: n where it is set, else 0
                            const float ln = __uint_as_float(__float_as_uint(n) & (unsigned)((int)__float_as_uint(nl[k]) >> 31));
                            y[k] = fmaf(p, mu[k], ln);
                            ks[u] = fmaf(ln, bias[g][k], fmaf(p, fmaf(mu[k], bias[g][k], fabsf(nl[k])), ks[u]));
                        }
                        av[u][g] = y;
                    }
                }
            };
            if (side) relu_step(std::true_type{});
            else relu_step(std::false_type{});
            if (it + 1 < ipp) fetch(cur, true, it + 1, X, PK);
            else fetch(nxt, nxt_live, 0, X, PK);
            if (t0 >= ntiles) continue;
            floatx16 acc[T][NT];
#pragma unroll
            for (int u = 0; u < T; ++u)
#pragma unroll
                for (int n = 0; n < NT; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[u][n][r] = 0.0f;
#pragma unroll
            for (int g = 0; g < CO8; ++g)
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                    for (int n = 0; n < NT; ++n)
#pragma unroll
                        for (int u = 0; u < T; ++u)
                            acc[u][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][g][s4], bk[n][4 * g + s4], acc[u][n], 0, 0, 0);
#pragma unroll
            for (int u = 0; u < T; ++u) {
                if (t0 + u >= ntiles) break;
                const float kt = ks[u] + __shfl_xor(ks[u], 32, 64);    // the two half-waves hold the two channel halves
                if (kq == 0) sK[(t0 + u) * 32 + l32] = kt;
#pragma unroll
                for (int n = 0; n < NT; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sP[((t0 + u) * 32 + 8 * (r >> 2) + 4 * kq + (r & 3)) * PS + n * 32 + l32] = acc[u][n][r];
            }
        }
        __syncthreads();

        // ---- gather the coefficients over the image and reduce them against the box ----
        const int total = a.RB * Pout, nky = (a.kh + S - 1) / S, nkx = (a.kw + S - 1) / S;
        const __amdgpu_buffer_rsrc_t lores = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(a.lo + (size_t)b * a.H * a.W * CI), 0, a.H * a.W * CI * 4, 0x00020000);
        const __amdgpu_buffer_rsrc_t hires = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(a.hi + (size_t)b * a.H * a.W * CI), 0, a.H * a.W * CI * 4, 0x00020000);
        for (int e = tid; e < total; e += kTailThreads) {
            const int ml = (int)(((unsigned long long)e * magic_pout) >> 32);
            const int q = e - ml * Pout;
            const int y = (int)(((unsigned long long)q * magic_ow) >> 32);
            const int x = q - y * a.ow;
            const int rbase = ml * npos;
            // both bounds of this position of the image are requested before the taps are gathered, so their latency
            // hides behind the LDS reads; a position off the image reads zeros (offset outside the resource)
            const int gy = qy + y, gx = qx + x;
            const int boff = (gy >= 0 && gy < a.H && gx >= 0 && gx < a.W) ? ((gy * a.W + gx) * CI) * 4 : (int)0x80000000;
            float blo[4] = {0.f, 0.f, 0.f, 0.f}, bhi[4] = {0.f, 0.f, 0.f, 0.f};
            if (a.RB > 0) {            // always true; inside a branch of their own the loads are not sunk to their use behind the loop
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (c < CI) {
                        blo[c] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(lores, boff + 4 * c, 0, 0));
                        bhi[c] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(hires, boff + 4 * c, 0, 0));
                    }
            }
            float o[4] = {0.f, 0.f, 0.f, 0.f};
            // taps that can reach this output: ky = y mod S + S * jy, read at patch row y / S - jy (same for x)
            const int ybase = y / S, ry = y - ybase * S, xbase = x / S, rx = x - xbase * S;
            for (int jy = 0; jy < nky; ++jy) {
                const int ky = ry + S * jy, py = ybase - jy;
                const bool oky = ky < a.kh && py >= 0 && py < a.ih;
                const int rowoff = rbase + py * a.iw;
                for (int jx = 0; jx < nkx; ++jx) {
                    const int kx = rx + S * jx, px = xbase - jx;
                    const bool ok = oky && kx < a.kw && px >= 0 && px < a.iw;
                    const float* src = sP + (ok ? (rowoff + px) * PS + (ky * a.kw + kx) * CI : zoff);
                    o[0] += src[0]; o[1] += src[1]; o[2] += src[2]; o[3] += src[3];      // columns past CI are not used
                }
            }
            float t = 0.0f;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c < CI) t = fmaf(o[c], (o[c] >= 0.0f) == (side == 0) ? blo[c] : bhi[c], t);
            sC[e] = t;
        }
        __syncthreads();

        // ---- per row: constant + ReLU-step contributions of its entries + box contributions of its positions ----
        for (int rbase = 0; rbase < a.RB; rbase += kTailThreads / 16) {
            const int r = rbase + (tid >> 4), k = tid & 15;
            float t = 0.0f;
            if (r < a.RB) {
                for (int q = r * npos + k; q < (r + 1) * npos; q += 16) t += sK[q];
                for (int q = r * Pout + k; q < (r + 1) * Pout; q += 16) t += sC[q];
            }
#pragma unroll
            for (int d = 8; d >= 1; d >>= 1) t += __shfl_xor(t, d, 64);
            if (k == 0 && r < a.RB && m0 + r < a.M) {
                const double c0 = SHARED ? (double)a.cst_init_c[co0 + r] : a.cst[m0 + r];
                (side == 0 ? a.out_l : a.out_u)[(size_t)b * a.R + r0 + r] = (float)(c0 + (double)t);
            }
        }
        __syncthreads();                   // the panel and the sums are overwritten by the next panel
        cur = nxt;
        cur_live = nxt_live;
    }
}

}  // namespace

bool launch_patch_tail(const PatchTail& d, hipStream_t s)
{
    const ConvGeom& g = *d.conv;
    if (conv_algo() != 0 || g.Ci > 4 || (g.stride != 1 && g.stride != 2) || g.kh * g.kw * g.Ci > 64) return false;
    if (g.Co != 8 && g.Co != 16 && g.Co != 32) return false;      // 64 channels would not fit the register file
    const PatchGeom& pg = *d.form;
    if (pg.C != g.Co || pg.gh != g.Ho || pg.gw != g.Wo || pg.rows_C < 1 || pg.rows_W < 1) return false;
    if (d.R < 1 || d.R % pg.rows_C != 0 || d.batch < 1 || d.ld_in % 4 != 0 || ((uintptr_t)d.in % 16) != 0 ||
        ((uintptr_t)d.pk2 % 16) != 0 || d.ldpk % 2 != 0 || d.ldpk < g.Co * g.Ho * g.Wo)
        return false;
    const int NT = (g.kh * g.kw * g.Ci + 31) / 32, PS = 32 * NT + 3;
    const int npos = pg.ph * pg.pw;
    const int oh = (pg.ph - 1) * g.stride + g.kh, ow = (pg.pw - 1) * g.stride + g.kw, Pout = oh * ow;
    // rows per panel: the largest power-of-two divisor of the channel count whose panel and sums fit 48 KB
    auto bytes = [&](int rb) {
        const size_t e32 = (size_t)round_up((int64_t)rb * npos, 32);
        return e32 * PS * 4 + 16 + e32 * 4 + (size_t)rb * Pout * 4;
    };
    int RB = 0;
    for (int rb = 1; rb <= 64 && pg.rows_C % rb == 0; rb *= 2)
        if (bytes(rb) <= 48 * 1024) RB = rb;
    if (RB == 0) return false;
    if ((int64_t)RB * d.ld_in * 4 >= ((int64_t)1 << 31) || (int64_t)d.ldpk * 8 >= ((int64_t)1 << 31)) return false;     // 32-bit buffer offsets
    const int64_t M = (int64_t)2 * d.batch * d.R;
    TailArgs a{};
    a.in = d.in; a.ld_in = d.ld_in; a.cst = d.cst; a.cst_init_c = d.cst_init_c;
    a.M = M; a.R = d.R; a.batch = d.batch; a.rows_W = pg.rows_W; a.rows_C = pg.rows_C;
    a.ih = pg.ph; a.iw = pg.pw; a.pS = pg.S; a.pP = pg.P; a.gh = pg.gh; a.gw = pg.gw;
    a.pk2 = reinterpret_cast<const float2*>(d.pk2); a.ldpk = d.ldpk; a.bias_c = d.bias_c;
    a.taps = d.taps; a.Ci = g.Ci; a.kh = g.kh; a.kw = g.kw;
    a.oh = oh; a.ow = ow; a.qS = pg.S * g.stride; a.qP = pg.P * g.stride + g.pad; a.H = g.H; a.W = g.W;
    a.lo = d.lo; a.hi = d.hi; a.out_l = d.out_l; a.out_u = d.out_u;
    a.RB = RB;
    const int64_t units = ceil_div(M, RB);
    a.panels = (int)std::max<int64_t>(1, std::min<int64_t>(16, units / 2048));
    const unsigned grid = (unsigned)ceil_div(units, a.panels);
    const size_t lds = bytes(RB);
    const bool shared = d.shared != 0;
    auto launch = [&](auto kern) { hipLaunchKernelGGL(kern, dim3(grid), dim3(kTailThreads), lds, s, a); };
#define DPC_TAIL_CASE(NTV, SV, C8)                                          \
    if (NT == NTV && g.stride == SV && g.Co == 8 * C8) {                    \
        if (shared) launch(&patch_tail_kernel<NTV, SV, C8, true>);          \
        else launch(&patch_tail_kernel<NTV, SV, C8, false>);                \
    }
    DPC_TAIL_CASE(1, 1, 1) DPC_TAIL_CASE(1, 1, 2) DPC_TAIL_CASE(1, 1, 4)
    DPC_TAIL_CASE(2, 1, 1) DPC_TAIL_CASE(2, 1, 2) DPC_TAIL_CASE(2, 1, 4)
    DPC_TAIL_CASE(1, 2, 1) DPC_TAIL_CASE(1, 2, 2) DPC_TAIL_CASE(1, 2, 4)
    DPC_TAIL_CASE(2, 2, 1) DPC_TAIL_CASE(2, 2, 2) DPC_TAIL_CASE(2, 2, 4)
#undef DPC_TAIL_CASE
    DPC_HIP(hipGetLastError());
    return true;
}

}  // namespace dpc
