// Transposed convolution of coefficient rows through a convolution layer (one traverse iteration
// when the bounds of the layer below are a Convolution block): fp32 MFMA implicit GEMM, and a
// plain-ALU kernel for layers with very few input channels (the image itself).
//
//   out[m, y, x, ci] = sum over taps (ky,kx) and channels co with (y+off-ky) = py*s, (x+off-kx) = px*s,
//                      0 <= py < ih, 0 <= px < iw, of in[m, py, px, co] * K[co, ci, ky, kx]
//
// Gather form: every output coefficient is produced by one accumulator, so the summation order is
// fixed and no atomics are needed.  With stride s the output positions fall into s*s parity classes
// (cy, cx) = ((y+off) mod s, (x+off) mod s); a class only meets the taps ky = cy (mod s), kx = cx
// (mod s), so inside a class the operation is a stride-1 correlation with a sub-sampled kernel.
//
// MFMA kernel (v_mfma_f32_32x32x2_f32): GEMM rows = 32 output positions of one class, taken from the
// flattened (row of the block, position) list so that small patches still fill whole tiles; GEMM
// columns = output channels ci; reduction = (tap, co).  A workgroup (4 wavefronts) owns up to 256
// list entries per class; each wavefront owns 2 position tiles x (Ci/32) channel tiles.  The input
// patches of the workgroup's rows sit in LDS ((H,W,C) order, position stride Co+4 floats to spread
// banks); a lane fetches the four consecutive channels it feeds with one 16-byte read at an address
// it computes from (position, tap), or from a zero block when the tap falls outside the patch.  When the
// patches of all channels would leave room for only one workgroup per CU, the reduction runs over channel
// chunks and LDS holds one chunk at a time.  Kernel values are read from global memory (L2-resident) one
// (tap, 8-channel group) ahead into registers, so the (tap, group) loop has no barrier.
#include <type_traits>

#include "conv.h"

namespace dpc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float vf4 __attribute__((ext_vector_type(4)));

constexpr int kCtThreads = 256;
constexpr int kCtEntries = 256;          // list entries per class per workgroup (4 waves x 2 tiles x 32)

struct CtArgs {
    const float* in; long long M; int ld_in; int ih, iw, Co;
    const float* taps; int Ci, kh, kw, s, off;      // conv_transpose_mfma_kernel: the [kh][kw][Co/4][Ci][4] layout
    float* out; int ld_out; int oh, ow;
    int RB;          // rows per workgroup
    int CC;          // channels of the reduction staged in LDS at a time (divides Co, multiple of 8)
    int pstride;     // LDS floats per input position (CC + 4)
    int rowstride;   // LDS floats per input row patch (ih*iw*pstride)
    // multiply-high constants 2^32 / d + 1 of the staging loops (d = CC / 4, ih * iw, iw), worked out on the host
    unsigned magic_cc4n, magic_npos, magic_iw;   // (0 for d = 1: the quotient is the dividend)
};

// RELU variants: the sign-split ReLU step of the layer above the convolution (with the bias fold of the convolution) is
// applied to the rows while their patches are staged in LDS; the constants it adds go to part[m] (one slot).
struct CtRelu {
    const float2* pk2; int ldpk;          // (mu, nu with lambda in the sign bit) [batch][ldpk], index (gy*gw + gx)*Co + c
    const float* bias_c;                  // [Co]
    float* part;                          // [M]
    int R, batch;                         // rows are [side][input][R]
    int patch, rows_C, rows_W, pS, pP;    // patch rows: origin of row r's patch = ((r/rows_C/rows_W)*pS - pP, ((r/rows_C)%rows_W)*pS - pP)
    int gh, gw;                           // grid of the ReLU layer
    int in_mod;                           // > 0: rows shared by all inputs and sides, row m reads input row m % in_mod
};

template <int NT, bool RELU>
__global__ __launch_bounds__(kCtThreads) void conv_transpose_mfma_kernel(CtArgs a, CtRelu rl)
{
    extern __shared__ float4 lds4[];
    float* sIn = reinterpret_cast<float*>(lds4);                       // [RB*rowstride] + zero block [pstride]
    const int in_floats = a.RB * a.rowstride;
    const int zoff = in_floats;                                        // zero block
    int4* sTab = reinterpret_cast<int4*>(sIn + in_floats + a.pstride); // [256] {e0, py0, px0, outoff}
    int* sOut = reinterpret_cast<int*>(sTab + kCtEntries);             // [256] outoff again, packed for 16-byte reads
    float* sRed = reinterpret_cast<float*>(sOut + kCtEntries);         // RELU: [RB][4] partial row constants

    // NT = 0: at most 16 input channels.  Tiles are then 16 entries x 16 channels (16x16x4 MFMA, four tiles per wavefront,
    // groups of 16 reduction channels) instead of 32 x 32 (32x32x2, two tiles, groups of 8): half of every 32-column
    // tile would be padding otherwise.
    constexpr bool HALF = NT == 0;
    constexpr int NTN = HALF ? 1 : NT;            // accumulators per tile
    constexpr int TT = HALF ? 4 : 2;              // tiles per wavefront
    constexpr int TE = HALF ? 16 : 32;            // list entries per tile
    constexpr int GC = HALF ? 16 : 8;             // reduction channels per (tap, group) step
    constexpr int AV = HALF ? 4 : 16;             // accumulator registers per tile
    using AccT = typename std::conditional<HALF, vf4, floatx16>::type;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & (TE - 1), kq = lane / TE;
    const long long m0 = (long long)blockIdx.x * a.RB;
    const int q0 = blockIdx.y * kCtEntries;
    // quotient and remainder by the stride (non-negative x): strides 1 and 2 take no division
    auto divs = [&](int x) __attribute__((always_inline)) { return a.s == 1 ? x : a.s == 2 ? x >> 1 : x / a.s; };
    auto mods = [&](int x) __attribute__((always_inline)) { return a.s == 1 ? 0 : a.s == 2 ? x & 1 : x % a.s; };
    const int npos = a.ih * a.iw;
    const int nchunks = a.Co / a.CC;                                   // channel chunks of the reduction
    const int cc4n = a.CC >> 2;
    // A single-row workgroup that is one of several entry blocks of its row reaches only a band of input rows (its 256
    // entries of every class cover a few output rows): only that band is staged.  With the ReLU step the first block
    // still stages everything, because it also adds up the row's constant.
    int band_lo = 0, band_n = npos;
    if (a.RB == 1 && gridDim.y > 1 && (!RELU || blockIdx.y > 0)) {
        int lo = a.ih, hi = -1;
        for (int cy = 0; cy < a.s; ++cy) {
            const int y0 = mods(cy + a.s * a.off - a.off);          // (cy - off) mod s, argument kept non-negative
            const int Hc = y0 < a.oh ? divs(a.oh - y0 + a.s - 1) : 0;
            const int base_y = divs(y0 + a.off - cy);
            const int nky = cy < a.kh ? divs(a.kh - cy + a.s - 1) : 0;
            for (int cx = 0; cx < a.s; ++cx) {
                const int x0 = mods(cx + a.s * a.off - a.off);
                const int Wc = x0 < a.ow ? divs(a.ow - x0 + a.s - 1) : 0;
                const int Pc = Hc * Wc;
                if (Pc == 0 || q0 >= Pc || nky == 0) continue;
                const int qe = min(q0 + kCtEntries, Pc) - 1;
                lo = min(lo, base_y + q0 / Wc - (nky - 1));
                hi = max(hi, base_y + qe / Wc);
            }
        }
        lo = max(lo, 0);
        hi = min(hi, a.ih - 1);
        band_lo = hi >= lo ? lo * a.iw : 0;
        band_n = hi >= lo ? (hi - lo + 1) * a.iw : 0;
    }
    const unsigned magic_cc4n = a.magic_cc4n;
    const unsigned magic_npos = band_n == npos ? a.magic_npos : band_n > 1 ? (unsigned)((1ull << 32) / (unsigned)band_n + 1) : 0u;
    auto quot = [](int x, unsigned magic) __attribute__((always_inline)) { return magic ? (int)__umulhi((unsigned)x, magic) : x; };

    // Staging reads go through buffer resources (offsets past the range return zeros: no branches around the loads) and
    // are issued kStageU at a time before the first LDS write, so a thread has several 16-byte loads in flight.
    constexpr int kStageU = 4, kStageR = 2;       // plain rows / rows with the ReLU step (four loads each)
    constexpr int kNoData = (int)0x80000000;
    const bool in_shared = RELU && rl.in_mod > 0;
    const long long rows_here = (a.M - m0 < a.RB) ? a.M - m0 : a.RB;
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(in_shared ? a.in : a.in + m0 * a.ld_in), 0, (int)((in_shared ? rl.in_mod : rows_here) * a.ld_in * 4), 0x00020000);

    const __amdgpu_buffer_rsrc_t ores =
        __builtin_amdgcn_make_buffer_rsrc(a.out + m0 * a.ld_out, 0, (int)(rows_here * a.ld_out * 4), 0x00020000);

    // stage channels [c0, c0 + CC) of the input patches of this workgroup's rows
    auto stage_input = [&](int c0) __attribute__((always_inline)) {
        const int total = a.RB * band_n * cc4n;
        for (int idx0 = tid; idx0 < total; idx0 += kCtThreads * kStageU) {
            vf4 v[kStageU];
            int dsto[kStageU];
#pragma unroll
            for (int u = 0; u < kStageU; ++u) {
                const int idx = idx0 + u * kCtThreads;
                // quotients by the run-time extents through multiply-high (exact: idx * divisor < 2^32)
                const int t = quot(idx, magic_cc4n), c4 = idx - t * cc4n;
                const int ml = quot(t, magic_npos), pos = band_lo + t - ml * band_n;
                const bool ok = idx < total;                       // rows past M lie past the resource's range
                v[u] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(
                                                   xres, ok ? (ml * a.ld_in + pos * a.Co + c0 + c4 * 4) * 4 : kNoData, 0, 0));
                dsto[u] = ok ? ml * a.rowstride + pos * a.pstride + c4 * 4 : -1;
            }
#pragma unroll
            for (int u = 0; u < kStageU; ++u)
                if (dsto[u] >= 0) *reinterpret_cast<vf4*>(sIn + dsto[u]) = v[u];
        }
    };

    // RELU staging: a wavefront takes a row at a time (4 / RB wavefronts share a row when the workgroup has fewer than four
    // rows), so a row's side, input and patch origin are scalars and its constant is one wavefront reduction in a fixed
    // order.  Positions off the layer's grid (zero padding: no neuron) are staged as zeros.
    const unsigned magic_iw = a.magic_iw;
    const __amdgpu_buffer_rsrc_t qres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float2*>(rl.pk2), 0, RELU ? rl.batch * rl.ldpk * 8 : 0, 0x00020000);
    auto stage_input_relu = [&](int c0) __attribute__((always_inline)) {
        const int span = band_n * cc4n;
        const int wpr = a.RB >= 4 ? 1 : a.RB == 2 ? 2 : a.RB == 1 ? 4 : 1, pw = wave % wpr;
        for (int ml = wave / wpr; ml < a.RB; ml += 4 / wpr) {
            const bool rowok = m0 + ml < a.M;
            const int m = rowok ? (int)(m0 + ml) : 0;                  // M < 2^31 (checked on the host)
            const int g = m / rl.R, r = m - g * rl.R;
            const bool upper_side = g >= rl.batch;
            const int b = g - (upper_side ? rl.batch : 0);
            int oy = 0, ox = 0;
            if (rl.patch) {
                const int wo = (r / rl.rows_C) % rl.rows_W, ho = r / (rl.rows_C * rl.rows_W);
                oy = ho * rl.pS - rl.pP;
                ox = wo * rl.pS - rl.pP;
            }
            const int xrow = ((in_shared ? m % rl.in_mod : ml) * a.ld_in + c0) * 4;     // bytes within xres
            const int qrow = (b * rl.ldpk + c0) * 8;                                     // bytes within qres
            float* dst = sIn + ml * a.rowstride;
            float acc = 0.0f;
            for (int i0 = pw * 64 + lane; i0 < span; i0 += 64 * wpr * kStageR) {
                vf4 x4[kStageR], p01[kStageR], p23[kStageR], b4[kStageR];
                int dsto[kStageR];
#pragma unroll
                for (int u = 0; u < kStageR; ++u) {
                    const int i = i0 + u * 64 * wpr;
                    const int pb = quot(i, magic_cc4n), c4 = i - pb * cc4n, pos = band_lo + pb;
                    const int py = quot(pos, magic_iw), px = pos - py * a.iw;
                    const int gy = oy + py, gx = ox + px;
                    const bool in = i < span;
                    const bool ok = in && rowok && gy >= 0 && gy < rl.gh && gx >= 0 && gx < rl.gw;
                    x4[u] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(
                                                        xres, ok ? xrow + (pos * a.Co + c4 * 4) * 4 : kNoData, 0, 0));
                    const int qo = ok ? qrow + ((gy * rl.gw + gx) * a.Co + c4 * 4) * 8 : kNoData;
                    p01[u] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(qres, qo, 0, 0));
                    p23[u] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(qres, qo, 16, 0));
                    b4[u] = *reinterpret_cast<const vf4*>(rl.bias_c + c0 + (in ? c4 * 4 : 0));
                    dsto[u] = in ? pos * a.pstride + c4 * 4 : -1;
                }
#pragma unroll
                for (int u = 0; u < kStageR; ++u) {
                    // off the grid or past the rows: x and the parameters read as zeros, so y = 0 and nothing is added
                    const float x[4] = {x4[u][0], x4[u][1], x4[u][2], x4[u][3]}, mu[4] = {p01[u][0], p01[u][2], p23[u][0], p23[u][2]};
                    const float nl[4] = {p01[u][1], p01[u][3], p23[u][1], p23[u][3]}, bs[4] = {b4[u][0], b4[u][1], b4[u][2], b4[u][3]};
                    vf4 y;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        // the part of x on which this side takes the upper relaxation is p, the rest n:
                        //   y = p * mu + lambda * n,   constant += p * (mu * bias + nu) + lambda * n * bias
                        const float p = upper_side ? fmaxf(x[k], 0.0f) : fminf(x[k], 0.0f);
                        const float n = x[k] - p;
                        const float ln = __uint_as_float(__float_as_uint(n) & (unsigned)((int)__float_as_uint(nl[k]) >> 31));
                        y[k] = fmaf(p, mu[k], ln);
                        acc = fmaf(ln, bs[k], fmaf(p, fmaf(mu[k], bs[k], fabsf(nl[k])), acc));
                    }
                    if (dsto[u] >= 0) *reinterpret_cast<vf4*>(dst + dsto[u]) = y;
                }
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
            if (lane == 0) sRed[ml * 4 + pw] = acc;
        }
    };
    // after the barrier behind a staging: the row constants of the staged channels, added once per row by the
    // workgroups with blockIdx.y == 0 while they stage for their first class
    bool consts_pending = RELU && blockIdx.y == 0;
    auto add_consts = [&](bool first_chunk) __attribute__((always_inline)) {
        if (!consts_pending) return;
        const int wpr = a.RB >= 4 ? 1 : a.RB == 2 ? 2 : a.RB == 1 ? 4 : 1;
        if (tid < a.RB && m0 + tid < a.M) {
            float t = 0.0f;
            for (int k = 0; k < wpr; ++k) t += sRed[tid * 4 + k];
            rl.part[m0 + tid] = first_chunk ? t : rl.part[m0 + tid] + t;
        }
    };

    for (int i = tid; i < a.pstride; i += kCtThreads) sIn[zoff + i] = 0.0f;
    if (blockIdx.y == 0) {           // padding columns of the output rows
        const int elems = a.oh * a.ow * a.Ci, padn = a.ld_out - elems;
        for (int i = tid; i < a.RB * padn; i += kCtThreads) {
            const int ml = i / padn, c = i - ml * padn;
            if (m0 + ml < a.M) a.out[(m0 + ml) * a.ld_out + elems + c] = 0.0f;
        }
    }
    if (nchunks == 1) {
        if constexpr (RELU) stage_input_relu(0);
        else stage_input(0);
    }
    __syncthreads();
    if (nchunks == 1) { add_consts(true); consts_pending = false; }

    // kernel values straight from global memory (the whole kernel is a few hundred KB and is read by every
    // workgroup, so it lives in L2): lane (kq, l32) needs K[tap][co = 8g+4kq+s][ci = 32n + l32], s = 0..3, which the
    // [tap][co / 4][ci][co % 4] layout holds in 16 consecutive bytes
    bool ci_ok[NTN];
    int kvoff[NTN];                                   // byte offset of this lane's kernel column (clamped into range)
#pragma unroll
    for (int n = 0; n < NTN; ++n) {
        ci_ok[n] = n * 32 + l32 < a.Ci;
        kvoff[n] = (kq * a.Ci + min(n * 32 + l32, a.Ci - 1)) * 16;
    }
    const __amdgpu_buffer_rsrc_t kres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.taps), 0, a.kh * a.kw * a.Co * a.Ci * 4, 0x00020000);

    for (int cy = 0; cy < a.s; ++cy) {
        // rows y of this class: (y + off) mod s == cy  ->  y = y0 + s*iy
        const int y0 = mods(cy + a.s * a.off - a.off);
        const int Hc = y0 < a.oh ? divs(a.oh - y0 + a.s - 1) : 0;
        const int base_y = divs(y0 + a.off - cy);
        const int nky = cy < a.kh ? divs(a.kh - cy + a.s - 1) : 0;
        for (int cx = 0; cx < a.s; ++cx) {
            const int x0 = mods(cx + a.s * a.off - a.off);
            const int Wc = x0 < a.ow ? divs(a.ow - x0 + a.s - 1) : 0;
            const int base_x = divs(x0 + a.off - cx);
            const int nkx = cx < a.kw ? divs(a.kw - cx + a.s - 1) : 0;
            const int Pc = Hc * Wc;
            if (Pc == 0 || q0 >= a.RB * Pc) continue;           // uniform over the workgroup

            // ---- table of this class's list entries ----
            {
                const float rPc = 1.0f / (float)Pc, rWc = 1.0f / (float)Wc;
                const int q = q0 + tid;
                int4 e = make_int4(0, 0, 0, -1);
                if (q < a.RB * Pc) {
                    // quotients through a float reciprocal with one correction step (exact: q < 2^22 on the host side)
                    int ml = (int)((float)q * rPc), pc = q - ml * Pc;
                    if (pc < 0) { --ml; pc += Pc; } else if (pc >= Pc) { ++ml; pc -= Pc; }
                    int iy = (int)((float)pc * rWc), ix = pc - iy * Wc;
                    if (ix < 0) { --iy; ix += Wc; } else if (ix >= Wc) { ++iy; ix -= Wc; }
                    if (m0 + ml < a.M) {
                        const int y = y0 + a.s * iy, x = x0 + a.s * ix;
                        e.x = ml * a.rowstride + ((base_y + iy) * a.iw + (base_x + ix)) * a.pstride;
                        e.y = base_y + iy;
                        e.z = base_x + ix;
                        e.w = ml * a.ld_out + (y * a.ow + x) * a.Ci;
                    }
                }
                sTab[tid] = e;
                sOut[tid] = e.w;
            }
            __syncthreads();

            int e0[TT], py0[TT], px0[TT];
            bool live[TT];
#pragma unroll
            for (int t = 0; t < TT; ++t) {
                const int4 e = sTab[wave * 64 + t * TE + l32];
                e0[t] = e.x + 4 * kq; py0[t] = e.y; px0[t] = e.z; live[t] = e.w >= 0;
            }
            AccT acc[TT][NTN];
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
                for (int n = 0; n < NTN; ++n)
#pragma unroll
                    for (int v = 0; v < AV; ++v) acc[t][n][v] = 0.0f;

            const int ntaps = nky * nkx;
            const int ngr = a.CC / GC;                            // groups of 8 (16) channels per chunk
            for (int cc = 0; cc < nchunks; ++cc) {
                if (nchunks > 1) {
                    __syncthreads();                              // everyone is done with the previous chunk
                    if constexpr (RELU) stage_input_relu(cc * a.CC);
                    else stage_input(cc * a.CC);
                    __syncthreads();
                    add_consts(cc == 0);
                }
                const int nit = ntaps * ngr;                      // flattened (tap, group) iterations
                // Kernel values through a buffer resource (one lane offset, scalar offsets for the rest), fetched three
                // (tap, group) steps ahead into rotating register sets.  Plain predicated pointer loads ended up in
                // separate basic blocks with a full wait behind them, which exposed the L2 latency at every step.
                // The loads and the steps each walk the (tap, group) sequence in order, so both keep running counters:
                // dividing the flattened index out again cost two scalar divisions per load and per step, ~120 scalar
                // instructions in front of every 8 (16) MFMAs.
                auto tap_off = [&](int jy, int jx) __attribute__((always_inline)) {
                    return (((cy + a.s * jy) * a.kw + (cx + a.s * jx)) * a.Co + cc * a.CC) * a.Ci * 4;   // bytes, wave-uniform
                };
                int lg = 0, ljx = 0, ljy = 0, lbase = tap_off(0, 0);      // (group, tap) of the next load
                auto load_b = [&](float (&bb)[4][NTN]) __attribute__((always_inline)) {
                    const int so = lbase + lg * GC * a.Ci * 4;
#pragma unroll
                    for (int n = 0; n < NTN; ++n) {
                        // columns past Ci read a clamped (valid) column: they only feed accumulator columns that
                        // are never stored, and touching the value here would force a wait right behind the load
                        const vf4 b4 = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(kres, kvoff[n], so, 0));
#pragma unroll
                        for (int s = 0; s < 4; ++s) bb[s][n] = b4[s];
                    }
                    if (++lg == ngr) {
                        lg = 0;
                        if (++ljx == nkx) { ljx = 0; ++ljy; }
                        lbase = tap_off(ljy, ljx);
                    }
                };
                int addr[TT];
#pragma unroll
                for (int t = 0; t < TT; ++t) addr[t] = zoff + 4 * kq;
                int sg = 0, sjx = 0, sjy = 0;                              // (group, tap) of the next step
                auto step = [&](float (&bb)[4][NTN]) __attribute__((always_inline)) {
                    const int g = sg;
                    if (g == 0) {
                        const int jy = sjy, jx = sjx;
#pragma unroll
                        for (int t = 0; t < TT; ++t) {
                            const int py = py0[t] - jy, px = px0[t] - jx;
                            // one select, no branches: unsigned compares fold the two range tests of each coordinate
                            const bool ok = live[t] & ((unsigned)py < (unsigned)a.ih) & ((unsigned)px < (unsigned)a.iw);
                            addr[t] = ok ? e0[t] - (jy * a.iw + jx) * a.pstride : zoff + 4 * kq;
                        }
                    }
                    float4 av[TT];
#pragma unroll
                    for (int t = 0; t < TT; ++t) av[t] = *reinterpret_cast<const float4*>(sIn + addr[t] + GC * g);
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int t = 0; t < TT; ++t) {
                            const float x = s == 0 ? av[t].x : s == 1 ? av[t].y : s == 2 ? av[t].z : av[t].w;
                            if constexpr (HALF) {
                                // lane (kq, l) holds A[entry l][k = kq] and B[k = kq][channel l]: k runs over channels 16g + 4kq + s
                                acc[t][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(x, bb[s][0], acc[t][0], 0, 0, 0);
                            } else {
#pragma unroll
                                for (int n = 0; n < NTN; ++n)
                                    acc[t][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, bb[s][n], acc[t][n], 0, 0, 0);
                            }
                        }
                    if (++sg == ngr) {
                        sg = 0;
                        if (++sjx == nkx) { sjx = 0; ++sjy; }
                    }
                };
                float b0[4][NTN], b1[4][NTN], b2[4][NTN], b3[4][NTN];
                if (nit > 0) load_b(b0);
                if (nit > 1) load_b(b1);
                if (nit > 2) load_b(b2);
                int it = 0;
                // full rounds of four steps while at least seven steps remain: no per-step bound checks
                for (; it + 7 <= nit; it += 4) {
                    load_b(b3); step(b0);
                    load_b(b0); step(b1);
                    load_b(b1); step(b2);
                    load_b(b2); step(b3);
                }
                for (; it < nit; it += 4) {
                    if (it + 3 < nit) load_b(b3);
                    step(b0);
                    if (it + 1 < nit) {
                        if (it + 4 < nit) load_b(b0);
                        step(b1);
                    }
                    if (it + 2 < nit) {
                        if (it + 5 < nit) load_b(b1);
                        step(b2);
                    }
                    if (it + 3 < nit) {
                        if (it + 6 < nit) load_b(b2);
                        step(b3);
                    }
                }
            }

            // ---- epilogue: accumulator register 4*i+j of a lane is list entry 8*i + 4*kq + j, channel l32 ----
            // Buffer stores: an entry past the list (offset -1) or a channel past Ci gets an offset outside the
            // resource and is dropped, so the epilogue has no branches; the offsets of four consecutive entries come
            // from one 16-byte LDS read.
            if constexpr (HALF) {
                // accumulator register i of a lane is list entry 4*kq + i of the tile, channel l
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const int4 o4 = *reinterpret_cast<const int4*>(sOut + wave * 64 + t * TE + 4 * kq);
                    const int oo[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        // through a VGPR of its own: with the accumulator element as the direct operand the compiler emitted
                        // the first register of the tile for all four stores
                        float v = acc[t][0][i];
                        asm volatile("" : "+v"(v));
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), ores,
                                                              oo[i] >= 0 && ci_ok[0] ? (oo[i] + l32) * 4 : kNoData, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int4 o4 = *reinterpret_cast<const int4*>(sOut + wave * 64 + t * 32 + 8 * i + 4 * kq);
                        const int oo[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
                        for (int j = 0; j < 4; ++j)
#pragma unroll
                            for (int n = 0; n < NT; ++n) {
                                float v = acc[t][n][4 * i + j];
                                asm volatile("" : "+v"(v));            // see above
                                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), ores,
                                                                      oo[j] >= 0 && ci_ok[n] ? (oo[j] + n * 32 + l32) * 4 : kNoData, 0, 0);
                            }
                    }
            }
            __syncthreads();          // the table is rebuilt by the next class
            if (nchunks > 1) consts_pending = false;              // every chunk has been staged once
        }
    }
}

// Few input channels (CI <= 4, e.g. the image): one thread per (row, output position), channel
// accumulators in registers.  Control flow is kept uniform (a tap that falls outside the patch reads
// a block of zeros instead of being skipped) and the kernel pointer is restrict-qualified, so the
// compiler keeps the kernel values in scalar registers: the inner loop is one 16-byte LDS read per
// 4*CI FMAs.
template <int CI>
__global__ __launch_bounds__(kCtThreads) void conv_transpose_smallci_kernel(
    const float* __restrict__ in, const float* __restrict__ taps, float* __restrict__ out, CtArgs a,
    int yrows_per_block, int lds_rows)
{
    extern __shared__ float4 lds4[];
    float* sIn = reinterpret_cast<float*>(lds4);
    const int tid = threadIdx.x;
    const long long m0 = (long long)blockIdx.x * a.RB;
    // output rows [yb, ye) of this block and the input rows [r_lo, r_hi) they can reach
    const int yb = blockIdx.y * yrows_per_block, ye = min(a.oh, yb + yrows_per_block);
    int r_lo = yb + a.off - (a.kh - 1);
    r_lo = r_lo <= 0 ? 0 : r_lo / a.s;
    const int r_hi = min(a.ih, (ye - 1 + a.off) / a.s + 1);
    const int nrows = max(0, r_hi - r_lo);                 // <= lds_rows by construction on the host
    const int c4n = a.Co >> 2, rowfl = lds_rows * a.iw * a.pstride;   // LDS floats per network row
    const int zoff = a.RB * rowfl;                                    // block of zeros [pstride]
    for (int idx = tid; idx < a.RB * nrows * a.iw * c4n; idx += kCtThreads) {
        const int c4 = idx % c4n, t = idx / c4n;
        const int pos = t % (nrows * a.iw), ml = t / (nrows * a.iw);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m0 + ml < a.M)
            v = *reinterpret_cast<const float4*>(in + (m0 + ml) * a.ld_in + ((size_t)r_lo * a.iw + pos) * a.Co + c4 * 4);
        *reinterpret_cast<float4*>(sIn + ml * rowfl + pos * a.pstride + c4 * 4) = v;
    }
    for (int i = tid; i < a.pstride; i += kCtThreads) sIn[zoff + i] = 0.0f;
    const int P = a.oh * a.ow, elems = P * CI, padn = a.ld_out - elems;
    if (blockIdx.y == 0)
        for (int i = tid; i < a.RB * padn; i += kCtThreads) {
            const int ml = i / padn, c = i - ml * padn;
            if (m0 + ml < a.M) out[(m0 + ml) * a.ld_out + elems + c] = 0.0f;
        }
    __syncthreads();
    const int span = (ye - yb) * a.ow, total = a.RB * span;
    for (int base = 0; base < total; base += kCtThreads) {
        const int e = base + tid;
        const int ml = e / span, p = yb * a.ow + (e - ml * span);
        const bool active = e < total && m0 + ml < a.M;
        const int y = p / a.ow, x = p - y * a.ow;
        float acc[CI];
#pragma unroll
        for (int c = 0; c < CI; ++c) acc[c] = 0.0f;
        for (int ky = 0; ky < a.kh; ++ky) {
            const int ty = y + a.off - ky;
            const int py = ty / a.s;
            const bool oky = active && ty >= 0 && py * a.s == ty && py < a.ih;
            for (int kx = 0; kx < a.kw; ++kx) {
                const int tx = x + a.off - kx;
                const int px = tx / a.s;
                const bool ok = oky && tx >= 0 && px * a.s == tx && px < a.iw;
                const float4* src = reinterpret_cast<const float4*>(
                    sIn + (ok ? ml * rowfl + ((py - r_lo) * a.iw + px) * a.pstride : zoff));
                const float* kt = taps + (size_t)(ky * a.kw + kx) * a.Co * CI;
#pragma unroll 2
                for (int c4 = 0; c4 < c4n; ++c4) {
                    const float4 v = src[c4];
                    const float xs[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int c = 0; c < CI; ++c) acc[c] = fmaf(xs[u], kt[(c4 * 4 + u) * CI + c], acc[c]);
                }
            }
        }
        if (active) {
            float* dst = out + (m0 + ml) * a.ld_out + (size_t)p * CI;
#pragma unroll
            for (int c = 0; c < CI; ++c) dst[c] = acc[c];
        }
    }
}


// Few input channels through the MFMA units: with CI <= 4 output channels per position a direct implicit GEMM
// would use 3 of the 32 columns of a tile.  Instead the per-position product with ALL taps is formed first,
//     P[(row, py, px)][(ky, kx), ci] = sum_co in[row, py, px, co] * K[co, ci, ky, kx]
// -- a GEMM with kh*kw*CI columns (27 of 32 for a 3x3 kernel on an RGB image, 48 of 64 for 4x4) -- into LDS, and
// every output coefficient then gathers its (at most kh*kw/s^2) terms from P in a fixed order.  The kernel matrix
// is read once per workgroup and kept in registers in the B-operand layout; input coefficients go from global
// memory straight into the A operand (a lane owns one list entry and reads its channels 16 bytes at a time;
// within each group of 8 channels the lower half-wave takes 0..3, the upper half 4..7), two tiles of 32 entries
// per wavefront in flight.  A workgroup walks `panels` consecutive panels (RB rows x one strip of output rows
// each) so that the kernel-matrix fetch and the launch cost are spread over more work.
constexpr int kPThreads = 256;         // workgroup of the product-then-gather kernel below

// RELU: the rows are dense rows over the first ReLU layer and its sign-split step (with the bias fold of the convolution
// below) is applied to them as they are loaded: stored value x * mult, row constant += x * k (see conv_tail.hip for
// the arithmetic).  Every strip of output rows adds the constants of the input rows it owns (a partition of the
// input rows) into its own slot, part[(slot0 + strip) * stride + m]; the consumer adds the slots in index order.
struct PRelu {
    const float2* pk2; int ldpk;          // (mu, nu with lambda in the sign bit) [batch][ldpk]
    const float* bias_c;                  // [CO]
    float* part; long long part_stride; int slot0;
    int R, batch;                         // rows are [side][input][R]; RB divides R
};

template <int NT, int S, int CO8, bool RELU>
__global__ __launch_bounds__(kPThreads) void conv_transpose_p_kernel(
    const float* __restrict__ in, const float* __restrict__ taps, float* __restrict__ out, CtArgs a,
    int yrows_per_block, int lds_rows, int panels, PRelu rl)
{
    constexpr int CO = CO8 * 8, NC = 32 * NT, PS = NC + 3, NW = kPThreads / 64;
    constexpr int TU = (RELU && CO8 >= 4) ? 1 : 2;      // tiles of 32 entries per wavefront per step (registers decide)
    extern __shared__ float4 lds4[];
    float* sP = reinterpret_cast<float*>(lds4);        // [entries rounded up to 32][PS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kq = lane >> 5;
    const int CI = a.Ci;
    const int yb = blockIdx.y * yrows_per_block, ye = min(a.oh, yb + yrows_per_block);
    int r_lo = yb + a.off - (a.kh - 1);
    r_lo = r_lo <= 0 ? 0 : (r_lo + S - 1) / S;                         // first input row any of these outputs reads
    const int r_hi = min(a.ih, (ye - 1 + a.off) / S + 1);
    const int nrows = max(0, r_hi - r_lo);                             // <= lds_rows by construction on the host
    const int ncols = a.kh * a.kw * CI;
    const int npos = nrows * a.iw, E = a.RB * npos, ntiles = (E + 31) >> 5;
    const int Pout = a.oh * a.ow, elems = Pout * CI, padn = a.ld_out - elems;
    const int span = (ye - yb) * a.ow, total = a.RB * span, nky = (a.kh + S - 1) / S, nkx = (a.kw + S - 1) / S;
    const unsigned long long magic_span = (1ull << 32) / (unsigned)max(span, 1) + 1;   // e / span for e * span < 2^32
    const unsigned long long magic_ow = (1ull << 32) / (unsigned)max(a.ow, 1) + 1;
    const int zoff = ((a.RB * lds_rows * a.iw + 31) & ~31) * PS;                         // four zeros behind the panel
    if (tid < 4) sP[zoff + tid] = 0.0f;
    float* sK = sP + zoff + 4;                         // RELU: [entries] row-constant contribution of every entry
    // input rows whose constants this strip adds: [own_lo, own_hi) partitions [0, ih) over the strips and lies
    // inside the rows the strip stages
    const int own_lo = blockIdx.y == 0 ? 0 : min(a.ih, (yb + a.off + S - 1) / S);
    const int own_hi = ye >= a.oh ? a.ih : min(a.ih, (ye + a.off + S - 1) / S);
    const unsigned long long magic_npos = (1ull << 32) / (unsigned)max(npos, 1) + 1;   // e / npos for e * npos < 2^32
    const unsigned long long magic_iw = (1ull << 32) / (unsigned)max(a.iw, 1) + 1;

    // kernel matrix in the B-operand layout: step (g, s4) of the reduction multiplies channel 8g + 4kq + s4
    float bk[NT][CO8 * 4];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int col = n * 32 + l32;
        const int tap = col / CI, ci = col - tap * CI;
#pragma unroll
        for (int k = 0; k < CO8 * 4; ++k) {
            const int co = 8 * (k >> 2) + 4 * kq + (k & 3);
            bk[n][k] = col < ncols ? taps[((size_t)tap * CO + co) * CI + ci] : 0.0f;
        }
    }

    // The input tiles of a wavefront are fetched one step ahead, across panel boundaries too, so that the loads of
    // the next step are in flight during the MFMAs of this one and during the gather phase.
    const int ipp = (ntiles + TU * NW - 1) / (TU * NW);                // steps per wavefront per panel
    constexpr int PU = RELU ? TU : 1, PG = RELU ? CO8 : 1;
    float bias[PG][4];                                 // RELU: convolution bias of this lane's channels
    if constexpr (RELU) {
#pragma unroll
        for (int g = 0; g < CO8; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k) bias[g][k] = rl.bias_c[8 * g + 4 * kq + k];
    }
    // Buffer loads: a lane outside the panel or the rows gets an offset outside the resource and reads zeros (no
    // branch, no zero fill); the resource starts at the panel's first row, so 32-bit offsets suffice.
    constexpr int kOutside = (int)0x80000000;
    auto fetch = [&](int pi, int it, vf4 (&r)[TU][CO8], float4 (&pk)[PU][PG][2], int (&own)[TU]) __attribute__((always_inline)) {
        const long long mraw = ((long long)blockIdx.x * panels + pi) * a.RB;
        const bool livep = pi < panels && mraw < a.M;
        const long long m0 = livep ? mraw : 0;
        const long long prow = a.M - m0 < a.RB ? a.M - m0 : a.RB;       // rows of this panel that exist
        const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(in + m0 * a.ld_in), 0, livep ? (int)(prow * a.ld_in * 4) : 0, 0x00020000);
        __amdgpu_buffer_rsrc_t qres = xres;
        if constexpr (RELU) {
            const int b = ((int)m0 / rl.R) % rl.batch;                 // RB divides R: one (side, input) group per panel; M < 2^31
            qres = __builtin_amdgcn_make_buffer_rsrc(const_cast<float2*>(rl.pk2 + (size_t)b * rl.ldpk), 0, livep ? rl.ldpk * 8 : 0,
                                                     0x00020000);
        }
        const int t0 = (wave + it * NW) * TU;
#pragma unroll
        for (int u = 0; u < TU; ++u) {
            const int e = (t0 + u) * 32 + l32;
            const int ml = (int)(((unsigned long long)e * magic_npos) >> 32), pos = e - ml * npos;
            const bool ok = t0 + u < ntiles && e < E;
            const int xo = ok ? (ml * a.ld_in + (r_lo * a.iw + pos) * CO + 4 * kq) * 4 : kOutside;
#pragma unroll
            for (int g = 0; g < CO8; ++g)
                r[u][g] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(xres, xo + 32 * g, 0, 0));
            if constexpr (RELU) {
                const int py = r_lo + (int)(((unsigned long long)pos * magic_iw) >> 32);
                own[u] = ok && py >= own_lo && py < own_hi;
                const int qo = ok ? ((r_lo * a.iw + pos) * CO + 4 * kq) * 8 : kOutside;
#pragma unroll
                for (int g = 0; g < CO8; ++g) {
                    pk[u][g][0] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(qres, qo + 64 * g, 0, 0));
                    pk[u][g][1] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(qres, qo + 64 * g + 16, 0, 0));
                }
            }
        }
    };
    vf4 nxt[TU][CO8];
    float4 npk[PU][PG][2];
    int nown[TU] = {};
    fetch(0, 0, nxt, npk, nown);

    for (int pi = 0; pi < panels; ++pi) {
        const long long m0 = ((long long)blockIdx.x * panels + pi) * a.RB;
        if (m0 >= a.M) break;                                          // uniform over the workgroup
        if (blockIdx.y == 0)
            for (int i = tid; i < a.RB * padn; i += kPThreads) {
                const int ml = i / padn, c = i - ml * padn;
                if (m0 + ml < a.M) out[(m0 + ml) * a.ld_out + elems + c] = 0.0f;
            }
        for (int it = 0; it < ipp; ++it) {
            const int t0 = (wave + it * NW) * TU;
            vf4 av[TU][CO8];
            if constexpr (RELU) {
                // per element x with (mu, nu | lambda) and the bias of its channel: the part of x on which this side takes the
                // upper relaxation is p (x >= 0 on the upper side, x < 0 on the lower side), the rest n:
                //   y = p * mu + lambda * n,   constant += p * (mu * bias + nu) + lambda * n * bias
                const bool upper_side = (int)m0 / rl.R >= rl.batch;
                float ks[TU] = {};
                auto relu_step = [&](auto up) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < TU; ++u)
#pragma unroll
                        for (int g = 0; g < CO8; ++g) {
                            const vf4 x = nxt[u][g];
                            const float4 p01 = npk[u][g][0], p23 = npk[u][g][1];
                            const float mu[4] = {p01.x, p01.z, p23.x, p23.z}, nl[4] = {p01.y, p01.w, p23.y, p23.w};
                            vf4 y;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const float p = decltype(up)::value ? fmaxf(x[k], 0.0f) : fminf(x[k], 0.0f);
                                const float n = decltype(up)::value ? fminf(x[k], 0.0f) : fmaxf(x[k], 0.0f);
                                const float ln = __uint_as_float(__float_as_uint(n) & (unsigned)((int)__float_as_uint(nl[k]) >> 31));
                                y[k] = fmaf(p, mu[k], ln);
                                ks[u] = fmaf(ln, bias[g][k], fmaf(p, fmaf(mu[k], bias[g][k], fabsf(nl[k])), ks[u]));
                            }
                            av[u][g] = y;
                        }
                };
                if (upper_side) relu_step(std::true_type{});
                else relu_step(std::false_type{});
#pragma unroll
                for (int u = 0; u < TU; ++u) {
                    const float kt = ks[u] + __shfl_xor(ks[u], 32, 64);     // the two half-waves hold the two channel halves
                    if (kq == 0 && t0 + u < ntiles) sK[(t0 + u) * 32 + l32] = nown[u] ? kt : 0.0f;
                }
            } else {
#pragma unroll
                for (int u = 0; u < TU; ++u)
#pragma unroll
                    for (int g = 0; g < CO8; ++g) av[u][g] = nxt[u][g];
            }
            if (it + 1 < ipp) fetch(pi, it + 1, nxt, npk, nown);
            else fetch(pi + 1, 0, nxt, npk, nown);
            if (t0 >= ntiles) continue;
            floatx16 acc[TU][NT];
#pragma unroll
            for (int u = 0; u < TU; ++u)
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
                        for (int u = 0; u < TU; ++u)
                            acc[u][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][g][s4], bk[n][4 * g + s4], acc[u][n], 0, 0, 0);
#pragma unroll
            for (int u = 0; u < TU; ++u) {
                if (t0 + u >= ntiles) break;
#pragma unroll
                for (int n = 0; n < NT; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sP[((t0 + u) * 32 + 8 * (r >> 2) + 4 * kq + (r & 3)) * PS + n * 32 + l32] = acc[u][n][r];
            }
        }
        __syncthreads();

        // Gather: one thread per output position, all taps in uniform control flow (a tap that falls outside the
        // patch reads a block of zeros); quotients by the run-time extents through multiply-high.
        for (int e = tid; e < total; e += kPThreads) {
            const int ml = (int)(((unsigned long long)e * magic_span) >> 32);
            const int q = e - ml * span;
            const int yy = (int)(((unsigned long long)q * magic_ow) >> 32);
            const int x = q - yy * a.ow, y = yb + yy;
            const int rbase = ml * npos - r_lo * a.iw;
            float o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
            // taps that can reach this output: ky = (y + off) mod S + S * jy, read at input row (y + off) / S - jy
            const int ybase = (y + a.off) / S, ry = y + a.off - ybase * S, xbase = (x + a.off) / S, rx = x + a.off - xbase * S;
            for (int jy = 0; jy < nky; ++jy) {
                const int ky = ry + S * jy, py = ybase - jy;
                const bool oky = ky < a.kh && py >= 0 && py < a.ih;
                const int rowoff = rbase + py * a.iw;
                for (int jx = 0; jx < nkx; ++jx) {
                    const int kx = rx + S * jx, px = xbase - jx;
                    const bool ok = oky && kx < a.kw && px >= 0 && px < a.iw;
                    const float* src = sP + (ok ? (rowoff + px) * PS + (ky * a.kw + kx) * CI : zoff);
                    o0 += src[0]; o1 += src[1]; o2 += src[2]; o3 += src[3];      // columns past CI are never stored
                }
            }
            if (m0 + ml < a.M) {
                float* dst = out + (m0 + ml) * a.ld_out + (size_t)(y * a.ow + x) * CI;
                dst[0] = o0;
                if (CI > 1) dst[1] = o1;
                if (CI > 2) dst[2] = o2;
                if (CI > 3) dst[3] = o3;
            }
        }
        if constexpr (RELU) {
            // per row: the contributions of its entries, 64 lanes of one wavefront per row, summed in a fixed order
            for (int ml = wave; ml < a.RB; ml += NW) {
                float t = 0.0f;
                for (int q = ml * npos + lane; q < (ml + 1) * npos; q += 64) t += sK[q];
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) t += __shfl_xor(t, d, 64);
                if (lane == 0 && m0 + ml < a.M) rl.part[(size_t)(rl.slot0 + blockIdx.y) * rl.part_stride + m0 + ml] = t;
            }
        }
        __syncthreads();                   // the panel is overwritten by the next one
    }
}

}  // namespace

// Returns false when the shape is outside what these kernels cover (the caller then uses the
// generic gather kernel).
bool launch_conv_transpose_fast(const float* in, int64_t M, int ld_in, int ih, int iw, const ConvGeom& g,
                                const ConvWeights& w, float* out, int ld_out, int oh, int ow, int off, hipStream_t s,
                                const ReluOnLoad* relu, int* slots_used)
{
    if (g.Co % 8 != 0 || ld_in % 4 != 0 || ((uintptr_t)in % 16) != 0) return false;
    if (relu && conv_algo() != 0) return false;
    if (relu && g.Ci <= 4 && (relu->form || relu->in_mod)) return false;   // few input channels: per-input dense rows only
    if (relu && (int64_t)ld_in < (int64_t)ih * iw * g.Co) return false;
    if ((int64_t)ld_in * 4 * 256 >= ((int64_t)1 << 31) || (int64_t)ld_out * 4 * 256 >= ((int64_t)1 << 31)) return false;
    if ((int64_t)oh * ow + kCtEntries >= ((int64_t)1 << 22)) return false;          // entry indices stay exact in fp32              // staging uses 32-bit byte offsets per workgroup
    if (relu && ((int64_t)relu->batch * relu->ldpk * 8 >= ((int64_t)1 << 31) || (int64_t)relu->in_mod * ld_in * 4 >= ((int64_t)1 << 31))) return false;
    CtArgs a{};
    a.in = in; a.M = M; a.ld_in = ld_in; a.ih = ih; a.iw = iw; a.Co = g.Co;
    a.taps = w.taps; a.Ci = g.Ci; a.kh = g.kh; a.kw = g.kw; a.s = g.stride; a.off = off;
    a.out = out; a.ld_out = ld_out; a.oh = oh; a.ow = ow;
    a.pstride = g.Co + 4;
    a.rowstride = ih * iw * a.pstride;
    constexpr size_t kLdsBudget = 150 * 1024;

    if (g.Ci <= 4 && conv_algo() != 2 && (g.stride == 1 || g.stride == 2) &&
        (g.Co == 8 || g.Co == 16 || g.Co == 32 || g.Co == 64) && g.kh * g.kw * g.Ci <= 64) {
        // MFMA route: P = input x all taps into LDS, then gather.  Workgroups take whole rows when the P panel of a
        // row fits (several rows if it is small), else strips of output rows.
        const int NT = (g.kh * g.kw * g.Ci + 31) / 32;
        const int PS = 32 * NT + 3;
        const size_t sB_bytes = 16;        // the block of zeros behind the panel
        // panel of at most 48 KB: three workgroups per compute unit, so that one's gather phase overlaps another's MFMAs
        // and loads (measured best among 24 .. 72 KB)
        const int64_t emax = (int64_t)((48 * 1024 - sB_bytes) / ((size_t)PS * 4)) / 32 * 32;     // list entries a panel can hold
        auto rows_reached = [&](int yb, int ye) {
            int r_lo = yb + off - (g.kh - 1);
            r_lo = r_lo <= 0 ? 0 : (r_lo + g.stride - 1) / g.stride;
            const int r_hi = std::min(ih, (ye - 1 + off) / g.stride + 1);
            return std::max(0, r_hi - r_lo);
        };
        int yr = oh, RB = 1, lds_rows = ih;
        if ((int64_t)ih * iw <= emax) {
            RB = (int)std::max<int64_t>(1, std::min<int64_t>(emax / ((int64_t)ih * iw), 64));
            if (relu) while (relu->R % RB != 0) --RB;                       // a panel stays inside one (side, input) group
        } else {
            for (yr = oh; yr >= 1; --yr) {
                lds_rows = 0;
                for (int yb = 0; yb < oh; yb += yr) lds_rows = std::max(lds_rows, rows_reached(yb, std::min(oh, yb + yr)));
                if ((int64_t)lds_rows * iw <= emax) break;
            }
        }
        const int strips = yr >= 1 ? (int)ceil_div(oh, yr) : 0;
        if (relu) {
            // every input row must be staged by some strip (its constants are added by the strip that owns it), the
            // strips need a slot each, and offsets must fit 32 bits
            const bool all_rows = (oh - 1 + off) / g.stride + 1 >= ih;
            if (!(yr >= 1 && (int64_t)RB * lds_rows * iw <= emax) || !all_rows || strips > relu->max_slots || M >= ((int64_t)1 << 31) ||
                (int64_t)RB * ld_in * 4 >= ((int64_t)1 << 31) || (int64_t)relu->ldpk * 8 >= ((int64_t)1 << 31) ||
                relu->ldpk < ih * iw * g.Co || ((uintptr_t)relu->pk2 % 16) != 0 || relu->part_stride < M)
                return false;
        }
        if (yr >= 1 && (int64_t)RB * lds_rows * iw <= emax) {
            a.RB = RB;
            const size_t e32 = (size_t)round_up((int64_t)RB * lds_rows * iw, 32);
            const size_t lds = sB_bytes + e32 * PS * 4 + (relu ? e32 * 4 : 0);
            // panels per workgroup: as many as keep about eight workgroups per compute unit in the grid
            const int64_t units = ceil_div(M, RB) * ceil_div(oh, yr);
            const int panels = (int)std::max<int64_t>(1, std::min<int64_t>(16, units / 2048));
            dim3 grid((unsigned)ceil_div(ceil_div(M, RB), panels), (unsigned)ceil_div(oh, yr));
            PRelu rl{};
            if (relu) {
                rl = PRelu{reinterpret_cast<const float2*>(relu->pk2), relu->ldpk, relu->bias_c, relu->part, relu->part_stride, 0, relu->R,
                           relu->batch};
                *slots_used = strips;
            }
            auto launch = [&](auto kern) {
                hipLaunchKernelGGL(kern, grid, dim3(kPThreads), lds, s, in, w.taps, out, a, yr, lds_rows, panels, rl);
            };
#define DPC_P_CASE(NTV, SV, C8) if (NT == NTV && g.stride == SV && g.Co == 8 * C8) { \
        if (relu) { \
            ensure_dynamic_lds(reinterpret_cast<const void*>(&conv_transpose_p_kernel<NTV, SV, C8, true>), 64 * 1024); \
            launch(&conv_transpose_p_kernel<NTV, SV, C8, true>); \
        } else { \
            ensure_dynamic_lds(reinterpret_cast<const void*>(&conv_transpose_p_kernel<NTV, SV, C8, false>), 64 * 1024); \
            launch(&conv_transpose_p_kernel<NTV, SV, C8, false>); \
        } }
            DPC_P_CASE(1, 1, 1) DPC_P_CASE(1, 1, 2) DPC_P_CASE(1, 1, 4) DPC_P_CASE(1, 1, 8)
            DPC_P_CASE(2, 1, 1) DPC_P_CASE(2, 1, 2) DPC_P_CASE(2, 1, 4) DPC_P_CASE(2, 1, 8)
            DPC_P_CASE(1, 2, 1) DPC_P_CASE(1, 2, 2) DPC_P_CASE(1, 2, 4) DPC_P_CASE(1, 2, 8)
            DPC_P_CASE(2, 2, 1) DPC_P_CASE(2, 2, 2) DPC_P_CASE(2, 2, 4) DPC_P_CASE(2, 2, 8)
#undef DPC_P_CASE
            DPC_HIP(hipGetLastError());
            return true;
        }
    }
    if (relu && g.Ci <= 4) return false;

    if (g.Ci <= 4) {
        // output rows per workgroup: about 256 positions; input rows those can reach: yr/s + (kh-1)/s + 2
        const int P = oh * ow;
        int yr = oh, RB = 1;
        if (P > 256) yr = std::max(1, 256 / ow);
        const int lds_rows = std::min(ih, (yr + g.stride - 1) / g.stride + (g.kh - 1) / g.stride + 2);
        const size_t rb_bytes = (size_t)lds_rows * iw * a.pstride * 4;
        if (P <= 256) RB = (int)std::max<int64_t>(1, std::min<int64_t>(256 / P, (int64_t)(48 * 1024 / rb_bytes)));
        if ((size_t)RB * rb_bytes + (size_t)a.pstride * 4 > kLdsBudget) return false;
        a.RB = RB;
        dim3 grid((unsigned)ceil_div(M, RB), (unsigned)ceil_div(oh, yr));
        const size_t lds = (size_t)RB * rb_bytes + (size_t)a.pstride * 4;
        auto launch = [&](auto kern) {
            ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kLdsBudget);
            hipLaunchKernelGGL(kern, grid, dim3(kCtThreads), lds, s, in, w.taps, out, a, yr, lds_rows);
        };
        switch (g.Ci) {
            case 1: launch(&conv_transpose_smallci_kernel<1>); break;
            case 2: launch(&conv_transpose_smallci_kernel<2>); break;
            case 3: launch(&conv_transpose_smallci_kernel<3>); break;
            default: launch(&conv_transpose_smallci_kernel<4>); break;
        }
        DPC_HIP(hipGetLastError());
        return true;
    }

    if (g.Ci > 64 || !w.taps4) return false;
    a.taps = w.taps4;
    // at most 16 input channels (and reduction channels in groups of 16): half-width tiles
    const bool half = g.Ci <= 16 && g.Co % 16 == 0 && conv_half_tiles() != 0;
    const int NT = half ? 0 : (g.Ci + 31) / 32;
    const int gc = half ? 16 : 8;
    // largest class decides how many rows fill the 256 list entries of a workgroup
    const int Pc_max = (int)(ceil_div(oh, g.stride) * ceil_div(ow, g.stride));
    int RB = std::max(1, kCtEntries / std::max(Pc_max, 1));
    // channel chunk: all channels if two workgroups then fit a CU, otherwise the largest divisor of Co that does
    int CC = g.Co;
    auto lds_for = [&](int rb, int cc) { return (size_t)rb * ih * iw * (cc + 4) * 4 + (size_t)(cc + 4) * 4 + 256 * 20 + (relu ? (size_t)rb * 16 : 0); };
    // two workgroups per CU with all channels staged at once when a workgroup holds several rows (measured: one chunk beats
    // two chunks at three workgroups per CU there); a single-row workgroup prefers the smaller chunk and three per CU
    const size_t cap = (RB >= 2 ? 77 : 72) * 1024;
    while (CC > gc && lds_for(RB, CC) > cap && (CC / 2) % gc == 0) CC /= 2;
    while (RB > 1 && lds_for(RB, CC) > cap) --RB;
    if (lds_for(RB, CC) > kLdsBudget) return false;
    a.CC = CC;
    a.pstride = CC + 4;
    a.rowstride = ih * iw * a.pstride;
    auto magic_of = [](int d) { return d > 1 ? (unsigned)((((uint64_t)1) << 32) / (unsigned)d + 1) : 0u; };
    a.magic_cc4n = magic_of(CC / 4);
    a.magic_npos = magic_of(ih * iw);
    a.magic_iw = magic_of(iw);
    const size_t row_bytes2 = (size_t)a.rowstride * 4;
    const size_t fixed = (size_t)a.pstride * 4 + 256 * 20 + (relu ? (size_t)RB * 16 : 0);
    a.RB = RB;
    CtRelu rl{};
    if (relu) {
        const int gh = relu->form ? relu->form->gh : ih, gw = relu->form ? relu->form->gw : iw;
        if (M >= ((int64_t)1 << 31) || relu->max_slots < 1 || relu->ldpk < gh * gw * g.Co || ((uintptr_t)relu->pk2 % 16) != 0 ||
            relu->part_stride < M || g.Co % 4 != 0 || relu->ldpk % 2 != 0 || ((uintptr_t)relu->bias_c % 16) != 0 || !relu->bias_c ||
            relu->R < 1 || relu->batch < 1 || relu->in_mod < 0 || (relu->in_mod > 0 && relu->R % relu->in_mod != 0) || (M != (int64_t)relu->R * relu->batch && M != 2 * (int64_t)relu->R * relu->batch) ||
            (relu->form && (relu->form->rows_C < 1 || relu->form->rows_W < 1 || relu->R % (relu->form->rows_C * relu->form->rows_W) != 0 ||
                            relu->form->C != g.Co || relu->form->ph != ih || relu->form->pw != iw)))
            return false;
        rl = CtRelu{reinterpret_cast<const float2*>(relu->pk2), relu->ldpk, relu->bias_c, relu->part, relu->R, relu->batch,
                    relu->form ? 1 : 0, relu->form ? relu->form->rows_C : 1, relu->form ? relu->form->rows_W : 1,
                    relu->form ? relu->form->S : 1, relu->form ? relu->form->P : 0, gh, gw, relu->in_mod};
        *slots_used = 1;
    }
    const size_t lds = (size_t)RB * row_bytes2 + fixed;
    dim3 grid((unsigned)ceil_div(M, RB), (unsigned)ceil_div((int64_t)RB * Pc_max, kCtEntries));
    auto launch = [&](auto kern) {
        ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kLdsBudget);
        hipLaunchKernelGGL(kern, grid, dim3(kCtThreads), lds, s, a, rl);
    };
    if (NT == 0) { if (relu) launch(&conv_transpose_mfma_kernel<0, true>); else launch(&conv_transpose_mfma_kernel<0, false>); }
    else if (NT == 1) { if (relu) launch(&conv_transpose_mfma_kernel<1, true>); else launch(&conv_transpose_mfma_kernel<1, false>); }
    else         { if (relu) launch(&conv_transpose_mfma_kernel<2, true>); else launch(&conv_transpose_mfma_kernel<2, false>); }
    DPC_HIP(hipGetLastError());
    return true;
}

}  // namespace dpc
