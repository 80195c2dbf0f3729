// Whole back-substitution of a fully-connected layer's rows in one kernel, coefficient rows resident in LDS.
//
// A traversal (backsubs_lower / backsubs_upper) of the R expressions of one (side, input) group touches, at
// every layer it crosses, only its own rows: row m of the coefficients over layer j-1 depends on row m over
// layer j alone.  A workgroup therefore takes BM rows of one group and walks them through every layer below
// without the coefficients ever leaving the compute unit:
//
//   fill   : rows of the layer's own weight matrix (shared by all inputs) go through the sign-split ReLU
//            step of the ReLU layer below (dense x diagonal) into the LDS panel sA[BM][width];
//   step j : acc = sA * W_j on the fp32 MFMA units (dense x dense; W_j streams from L2 straight into
//            registers -- every wavefront owns distinct output columns, so staging W_j through LDS would
//            share nothing); the accumulators go through the next ReLU step and overwrite sA;
//   last   : acc = sA * W_1, reduced against the input box (concretisation); nothing is stored.
//
// Row constants (nu and bias terms, finally the box term) are summed per step in fp32 over the columns, in a
// fixed order, and accumulated per row in fp64 in LDS.  The packed per-(group, column) parameters
// (pm, nm, kp, kn) are the ones the per-layer fused contraction uses: stored value x * (x >= 0 ? pm : nm),
// constant += x * (x >= 0 ? kp : kn).
//
// gfx950: 160 KB of LDS hold 64 rows of up to 512 coefficients (or 32 rows of up to 1024); 8 wavefronts,
// two per SIMD; v_mfma_f32_32x32x2_f32.  Operand layouts of that instruction: lane l feeds A[row l%32][k l/32]
// and B[k l/32][col l%32]; accumulator register 4i+j of lane l is row 8i + 4(l/32) + j, column l%32.  Within
// each group of 8 k the lower half-wave takes k 0..3 and the upper half k 4..7, so that a lane reads its four
// A values with one 16-byte LDS read; MFMA step s of the group multiplies k = {s, 4+s}.
#include <algorithm>

#include "common.h"

namespace dpc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float vf4 __attribute__((ext_vector_type(4)));

constexpr int kChainMaxSteps = 14;

struct ChainStep {
    const float* W;        // [round_up(K, 8)][ldw], rows K.. and columns past the layer's inputs are zero
    const float4* pk;      // packed parameters of the step that follows this contraction: [groups][ldpk]
    int K;                 // width of the expressions entering the step (rows of W)
    int ldw;               // multiple of 32: the step produces ldw / 32 column blocks
    int ldpk;              // >= ldw
    int store;             // 1: the result becomes the next panel; 0: concretisation, constants only
};

struct ChainArgs {
    const float* W0;       // the bounded layer's own rows [R][ldw0] (zero padded columns)
    const float* bias0;    // [R]
    const float4* pk0;     // packed parameters of the ReLU layer directly below: [groups][ldpk0]
    int ldw0, ldpk0;
    int width0;            // multiple of 32, <= KMAX: columns of the initial panel
    int R, B, bpg;         // rows per group, inputs, workgroups per group
    int nsteps;
    float* out_l;          // [B][R]
    float* out_u;          // [B][R]
    ChainStep step[kChainMaxSteps];
};

// One contraction step for a wavefront that owns MB row blocks (rows mrow .. mrow + 32*MB - 1 of the panel)
// and NA column blocks (blocks nb0 + nbs*q, q < NA), followed by the traversal step in registers.
template <int BM, int LDA, int MB, int NA, int WN>
__device__ __forceinline__ void chain_step(float* __restrict__ sA, double* __restrict__ sCst, float* __restrict__ sPart,
                                           const ChainStep& S, int g, int mrow, int wn, int nb0, int nbs, int lane, int tid)
{
    const int l32 = lane & 31, kq = lane >> 5;
    constexpr int NB = NA > 0 ? NA : 1;
    constexpr int PF = NA <= 4 ? 2 : 1;          // K groups of W kept in flight ahead of the one being multiplied
    float rs[MB][16];

    if constexpr (NA > 0) {
        floatx16 acc[MB][NB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < NB; ++q)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[mb][q][e] = 0.0f;

        const int nkg = (S.K + 7) >> 3;
        const unsigned lane_off = (unsigned)(4 * kq * S.ldw + nb0 * 32 + l32);
        const float* pa = sA + (mrow + l32) * LDA + 4 * kq;

        float4 P[NB];
        if constexpr (NA <= 4) {
#pragma unroll
            for (int q = 0; q < NB; ++q) P[q] = S.pk[(size_t)g * S.ldpk + (nb0 + nbs * q) * 32 + l32];
        }

        float b0[4][NB], b1[4][NB], b2[4][NB];      // K groups kg, kg+1, (kg+2) of W: the buffer a body consumes is refilled
                                                    // at once with the group PF+1 ahead, so no value is ever copied
        vf4 ac[MB], an[MB];
        // W is read through a buffer resource: one lane offset in a VGPR, everything else in scalar offsets.
        // (Plain pointer loads of values that are only used iterations later get sunk by the compiler down to
        // their use, which undoes the software pipeline.)
        const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(S.W), 0, ((S.K + 7) & ~7) * S.ldw * 4, 0x00020000);
        const int voff = (int)lane_off * 4;
        auto load_b = [&](float (&dst)[4][NB], int kg) __attribute__((always_inline)) {
            const int srow = kg * 8 * S.ldw * 4;
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int q = 0; q < NB; ++q)
                    dst[s][q] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(wres, voff + q * nbs * 128, srow + s * S.ldw * 4, 0));
        };
        auto load_a = [&](vf4 (&dst)[MB], int kg) __attribute__((always_inline)) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) dst[mb] = *reinterpret_cast<const vf4*>(pa + mb * 32 * LDA + kg * 8);
        };
        const int last = nkg - 1;
        load_b(b0, 0);
        load_b(b1, 1 < last ? 1 : last);
        if constexpr (PF == 2) load_b(b2, 2 < last ? 2 : last);
        load_a(ac, 0);
        // (prefetch indices are clamped: the last groups are fetched again rather than reading past W)
        auto body = [&](float (&bx)[4][NB], int kg) __attribute__((always_inline)) {
            const int ka = kg + 1;
            load_a(an, ka < last ? ka : last);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int q = 0; q < NB; ++q)
                        acc[mb][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(ac[mb][s], bx[s][q], acc[mb][q], 0, 0, 0);
            const int kf = kg + 1 + PF;
            load_b(bx, kf < last ? kf : last);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) ac[mb] = an[mb];
        };
        int kg = 0;
        if constexpr (PF == 2) {
            for (; kg + 3 <= nkg; kg += 3) { body(b0, kg); body(b1, kg + 1); body(b2, kg + 2); }
            if (kg < nkg) body(b0, kg);
            if (kg + 1 < nkg) body(b1, kg + 1);
        } else {
            for (; kg + 2 <= nkg; kg += 2) { body(b0, kg); body(b1, kg + 1); }
            if (kg < nkg) body(b0, kg);
        }

        if constexpr (NA > 4) {
#pragma unroll
            for (int q = 0; q < NB; ++q) P[q] = S.pk[(size_t)g * S.ldpk + (nb0 + nbs * q) * 32 + l32];
        }

        __syncthreads();                          // every wavefront is done reading the panel
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = mrow + mb * 32 + 8 * (e >> 2) + 4 * kq + (e & 3);
                float sum = 0.0f;
#pragma unroll
                for (int q = 0; q < NB; ++q) {
                    const float x = acc[mb][q][e];
                    const bool pos = x >= 0.0f;
                    sum += x * (pos ? P[q].z : P[q].w);
                    if (S.store) sA[row * LDA + (nb0 + nbs * q) * 32 + l32] = x * (pos ? P[q].x : P[q].y);
                }
                rs[mb][e] = sum;
            }
    } else {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) rs[mb][e] = 0.0f;
        __syncthreads();
    }

    // Row sums over the 32 lanes that share these rows: butterfly with halving.  After the steps with lane
    // bits 0..3 a lane holds the sum over its 16-lane group of register index 8*b0 + 4*b1 + 2*b2 + b3; the
    // last step adds the two groups.
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        float v8[8], v4[4], v2[2], v1;
        {
            const bool h = l32 & 1;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float send = h ? rs[mb][k] : rs[mb][k + 8];
                const float keep = h ? rs[mb][k + 8] : rs[mb][k];
                v8[k] = keep + __shfl_xor(send, 1, 64);
            }
        }
        {
            const bool h = l32 & 2;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float send = h ? v8[k] : v8[k + 4];
                const float keep = h ? v8[k + 4] : v8[k];
                v4[k] = keep + __shfl_xor(send, 2, 64);
            }
        }
        {
            const bool h = l32 & 4;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const float send = h ? v4[k] : v4[k + 2];
                const float keep = h ? v4[k + 2] : v4[k];
                v2[k] = keep + __shfl_xor(send, 4, 64);
            }
        }
        {
            const bool h = l32 & 8;
            const float send = h ? v2[0] : v2[1];
            const float keep = h ? v2[1] : v2[0];
            v1 = keep + __shfl_xor(send, 8, 64);
        }
        v1 += __shfl_xor(v1, 16, 64);
        if (l32 < 16) {
            const int v = 8 * (l32 & 1) + 4 * ((l32 >> 1) & 1) + 2 * ((l32 >> 2) & 1) + ((l32 >> 3) & 1);
            sPart[wn * BM + mrow + mb * 32 + 8 * (v >> 2) + 4 * kq + (v & 3)] = v1;
        }
    }
    __syncthreads();
    if (tid < BM) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < WN; ++w) t += sPart[w * BM + tid];
        sCst[tid] += (double)t;
    }
}

// BM rows per workgroup, KMAX = widest panel; (MBS, NBS): row blocks per wavefront and the most column blocks
// per wavefront in the steps that store a panel; (MBF, NBF): the same for the last step, whose columns (the
// network's inputs) are dealt to the wavefronts in chunks of WNF * NBF blocks.
template <int BM, int KMAX, int WAVES, int MBS, int NBS, int MBF, int NBF>
__global__ __launch_bounds__(WAVES * 64, 2) void chain_kernel(ChainArgs a)
{
    constexpr int LDA = KMAX + 4;                 // row stride = 4 banks: conflict-free 16-byte reads down a column of rows
    constexpr int WMS = BM / 32 / MBS, WNS = WAVES / WMS;
    constexpr int WMF = BM / 32 / MBF, WNF = WAVES / WMF;
    static_assert(WMS * MBS * 32 == BM && WMF * MBF * 32 == BM && WNS >= 1 && WNF >= 1, "wave layout");
    extern __shared__ float4 lds4[];
    float* sA = reinterpret_cast<float*>(lds4);                       // [BM][LDA]
    double* sCst = reinterpret_cast<double*>(sA + BM * LDA);          // [BM]
    float* sPart = reinterpret_cast<float*>(sCst + BM);               // [WAVES][BM]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.x / a.bpg;
    const int r0 = (blockIdx.x - g * a.bpg) * BM;

    // ---- fill: own rows through the ReLU step directly below ----
    // Every row of the workgroup belongs to the same (side, input) group: a lane keeps the parameters of its
    // columns in registers and streams the weight rows past them.
    {
        constexpr int NT = KMAX / 256;
        float4 P[NT][4];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int c = lane * 4 + 256 * t;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                P[t][k] = c < a.width0 ? a.pk0[(size_t)g * a.ldpk0 + c + k] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int r = wave; r < BM; r += WAVES) {
            const bool rv = r0 + r < a.R;
            const float* src = a.W0 + (size_t)(rv ? r0 + r : 0) * a.ldw0;
            vf4 x[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int c = lane * 4 + 256 * t;
                x[t] = vf4{0.f, 0.f, 0.f, 0.f};
                if (rv && c < a.width0) x[t] = *reinterpret_cast<const vf4*>(src + c);
            }
            float sum = 0.0f;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int c = lane * 4 + 256 * t;
                vf4 o;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool pos = x[t][k] >= 0.0f;
                    o[k] = x[t][k] * (pos ? P[t][k].x : P[t][k].y);
                    sum += x[t][k] * (pos ? P[t][k].z : P[t][k].w);
                }
                if (c < a.width0) *reinterpret_cast<vf4*>(sA + r * LDA + c) = o;
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
            if (lane == 0) sCst[r] = rv ? (double)a.bias0[r0 + r] + (double)sum : 0.0;
        }
    }
    __syncthreads();

    for (int st = 0; st < a.nsteps; ++st) {
        const ChainStep& S = a.step[st];
        const int nblk = S.ldw >> 5;
        if (S.store) {
            const int wm = wave / WNS, wn = wave - wm * WNS;
            const int left = nblk - wn;
            const int nact = left <= 0 ? 0 : (left + WNS - 1) / WNS;
            const int mrow = wm * MBS * 32;
#define DPC_CHAIN_CASE(NA)                                                                                         \
    case NA:                                                                                                       \
        if constexpr (NA <= NBS) chain_step<BM, LDA, MBS, NA, WNS>(sA, sCst, sPart, S, g, mrow, wn, wn, WNS, lane, tid); \
        break;
            switch (nact) {
                DPC_CHAIN_CASE(0) DPC_CHAIN_CASE(1) DPC_CHAIN_CASE(2) DPC_CHAIN_CASE(3) DPC_CHAIN_CASE(4)
                default: break;        // the host never launches a shape with more column blocks per wavefront
            }
#undef DPC_CHAIN_CASE
        } else {
            // Column blocks are dealt round-robin to the wavefronts, so the first ones get one more when the count
            // does not divide.  Wavefronts w and w + 4 share a SIMD, and so do equal wavefronts of two workgroups
            // on one compute unit: the dealing direction alternates with the row block and the workgroup so that
            // the extra blocks land on different SIMDs.
            const int wm = wave / WNF, wnp = wave - wm * WNF;
            const int wn = ((blockIdx.x + wm) & 1) ? WNF - 1 - wnp : wnp;
            const int mrow = wm * MBF * 32;
            for (int base = 0; base < nblk; base += WNF * NBF) {
                const int left = nblk - base - wn;
                int nact = left <= 0 ? 0 : (left + WNF - 1) / WNF;
                if (nact > NBF) nact = NBF;
#define DPC_CHAIN_CASE(NA)                                                                                         \
    case NA:                                                                                                       \
        if constexpr (NA <= NBF) chain_step<BM, LDA, MBF, NA, WNF>(sA, sCst, sPart, S, g, mrow, wn, base + wn, WNF, lane, tid); \
        break;
                switch (nact) {
                    DPC_CHAIN_CASE(0) DPC_CHAIN_CASE(1) DPC_CHAIN_CASE(2) DPC_CHAIN_CASE(3) DPC_CHAIN_CASE(4)
                    DPC_CHAIN_CASE(5) DPC_CHAIN_CASE(6) DPC_CHAIN_CASE(7)
                    default: break;
                }
#undef DPC_CHAIN_CASE
            }
        }
    }

    // sCst[tid] was last written by this same thread
    if (tid < BM && r0 + tid < a.R) {
        const int side = g / a.B, b = g - side * a.B;
        float* out = side == 0 ? a.out_l : a.out_u;
        out[(size_t)b * a.R + r0 + tid] = (float)sCst[tid];
    }
}

template <int BM, int KMAX, int WAVES>
constexpr size_t chain_lds_bytes() { return (size_t)BM * (KMAX + 4) * 4 + (size_t)BM * 8 + (size_t)WAVES * BM * 4; }


template <int BM, int KMAX, int WAVES, int MBS, int NBS, int MBF, int NBF>
void launch_chain_variant(const ChainArgs& a, int groups, hipStream_t s)
{
    constexpr size_t lds = chain_lds_bytes<BM, KMAX, WAVES>();
    ensure_dynamic_lds(reinterpret_cast<const void*>(&chain_kernel<BM, KMAX, WAVES, MBS, NBS, MBF, NBF>), (int)lds);
    hipLaunchKernelGGL((chain_kernel<BM, KMAX, WAVES, MBS, NBS, MBF, NBF>), dim3((unsigned)(groups * a.bpg)), dim3(WAVES * 64), lds,
                       s, a);
    DPC_HIP(hipGetLastError());
}

}  // namespace


// See common.h.  Returns false (nothing launched) when the shape is not covered or not worth it.
bool launch_chain(const ChainDesc& d, hipStream_t s)
{
    DPC_REQUIRE(d.W0 && d.bias0 && d.pk0 && d.out_l && d.out_u && d.nsteps >= 1 && d.steps, DPC_EINVAL, "chain: bad arguments");
    // tuning "chain": -1 by shape, 0 never, 1 whenever the shape is covered; "chain_rows": row block of the variant for
    // panels up to 512 columns, 64 or 32 (two workgroups per CU)
    const int g_chain = tune(TK_CHAIN), g_chain_rows = tune(TK_CHAIN_ROWS) == 32 ? 32 : 64;
    if (g_chain == 0 || d.nsteps > kChainMaxSteps || d.R < 1 || d.B < 1) return false;
    // widths: every panel (the initial one and the output of every storing step) and every K
    int wmax = d.width0;
    for (int i = 0; i < d.nsteps; ++i) {
        const ChainStepDesc& t = d.steps[i];
        if (!t.W || !t.pk || t.K < 1 || t.ldw % 32 != 0 || t.ldpk < t.ldw) return false;
        if ((i == d.nsteps - 1) != (t.store == 0)) return false;            // exactly the last step concretises
        if (t.K > (i == 0 ? d.width0 : d.steps[i - 1].ldw)) return false;   // K columns must exist in the panel
        if (t.store) wmax = std::max(wmax, t.ldw);
        if (((uintptr_t)t.W % 16) != 0 || ((uintptr_t)t.pk % 16) != 0) return false;
    }
    if (d.width0 % 32 != 0 || d.ldw0 < d.width0 || d.ldw0 % 4 != 0 || d.ldpk0 < d.width0) return false;
    if (((uintptr_t)d.W0 % 16) != 0 || ((uintptr_t)d.pk0 % 16) != 0) return false;
    int dev = 0, lds_max = 0;
    DPC_HIP(hipGetDevice(&dev));
    DPC_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    const int groups = 2 * d.B;
    const bool small = wmax <= 512;
    if (!small && wmax > 1024) return false;
    // Panels up to 512 columns: 32 rows and 4 wavefronts per workgroup, two workgroups per compute unit (one
    // hides the other's fill, epilogues and pipeline ramps); or 64 rows and 8 wavefronts, one per unit.  Wider
    // panels: 32 rows, 8 wavefronts, one workgroup per unit.
    const int BM = small ? g_chain_rows : 32;
    const size_t lds = !small ? chain_lds_bytes<32, 1024, 8>() : BM == 64 ? chain_lds_bytes<64, 512, 8>() : chain_lds_bytes<32, 512, 4>();
    if ((size_t)lds_max < lds) return false;
    const int bpg = (int)ceil_div(d.R, BM);
    if ((int64_t)groups * bpg > (1 << 30)) return false;
    if (g_chain < 0) {
        // by shape: enough workgroups to occupy the 256 compute units, row blocks mostly full
        const int64_t resident = (small && BM == 32) ? 512 : 256;
        if ((int64_t)groups * bpg < resident - resident / 8 || (double)d.R / ((double)bpg * BM) < 0.7) return false;
    }
    ChainArgs a{};
    a.W0 = d.W0; a.bias0 = d.bias0; a.pk0 = reinterpret_cast<const float4*>(d.pk0);
    a.ldw0 = d.ldw0; a.ldpk0 = d.ldpk0; a.width0 = d.width0;
    a.R = d.R; a.B = d.B; a.bpg = bpg; a.nsteps = d.nsteps;
    a.out_l = d.out_l; a.out_u = d.out_u;
    for (int i = 0; i < d.nsteps; ++i) {
        const ChainStepDesc& t = d.steps[i];
        a.step[i] = ChainStep{t.W, reinterpret_cast<const float4*>(t.pk), t.K, t.ldw, t.ldpk, t.store};
    }
    if (!small) launch_chain_variant<32, 1024, 8, 1, 4, 1, 4>(a, groups, s);
    else if (BM == 64) launch_chain_variant<64, 512, 8, 2, 2, 1, 7>(a, groups, s);
    else launch_chain_variant<32, 512, 4, 1, 4, 1, 7>(a, groups, s);
    return true;
}

}  // namespace dpc
