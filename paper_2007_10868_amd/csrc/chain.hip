// Fused back-substitution of a chain of narrow dense layers: ONE launch per start layer.
//
// Paper Section 2 ("Bottleneck Backsubstitution"): the rows of a start layer are independent, and a row's
// back-substitution is a fixed sequence of steps (ReLU substitution, product with the next layer's matrix, candidate
// bound).  For a network of narrow dense layers (a few hundred neurons) every one of these steps is a launch of a few
// microseconds when run on its own, and a pass is some 150 dependent launches.  Here a work-group takes 8 neurons of
// the start layer (16 rows: the expressions of +x and of -x) and carries them through ALL steps down to the input:
// the rows' coefficient block never leaves LDS, the layers' matrices (a few hundred KB in total) are
// streamed from L2, the products run on the float64 matrix instruction, and the per-row sums of the candidate bounds are
// taken from LDS right after each product.  The arithmetic of a step is that of the unfused kernels: one float32
// coefficient per entry, float64 accumulation, one rounding, the same slack terms (device_common.hpp).
#include "device_common.hpp"

namespace gp {

namespace {

constexpr int CH_ROWS = 16;          // rows per work-group: 8 tasks x {+x, -x}
constexpr int CH_TASKS = 8;
constexpr int CH_WAVES = 8;          // one wave per task in the row sums; two waves per SIMD hide each other's latencies
constexpr int CH_THREADS = 64 * CH_WAVES;
static_assert(CH_WAVES == CH_TASKS, "the row sums and the initial block give every task a wave of its own");

// out[16][n] = in[16][K] * W^T for the dense layer with matrix w[n][K], times the ReLU substitution of the
// destination layer, rounded once to float32.  in/out: LDS, row strides si/so (floats); the columns of `in` from K up to
// the next multiple of 16 are zero; out is written up to the next multiple of 16 of n (zeros beyond n).
// FR: column fragments (16 columns each) a wave works on together (1 for narrow layers, so that every wave of the
// work-group has a group of its own).  The matrix comes from L2 or beyond, one to two microseconds away, and there is
// little arithmetic per byte at 16 rows: what counts is how many bytes a wave has in flight.  So the float32 weights are
// read (half the bytes of the float64 copy; the conversions are cheap here) and a wave requests its columns' values
// for 8 chunks of 16 k (all of K up to 128) before the first product.
template <bool VEC, int FR>
__device__ __forceinline__ void chain_cross(const ChainStep& st, const float* in, int si, float* out, int so,
                                            const int* s_box) {
    constexpr int D = FR == 4 ? 7 : 8;      // (four fragments of 8 chunks each would spill)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lk = lane >> 4, lm = lane & 15;
    const int K = st.K, N = st.n;
    const int kchunks = (K + 15) >> 4;
    const int nfrag = (N + 15) >> 4;
    const int ngroups = (nfrag + FR - 1) / FR;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)st.w, 0, (int)((uint32_t)N * (uint32_t)K * 4u), 0x00020000);
    for (int g = wave; g < ngroups; g += CH_WAVES) {
        double4_t acc[FR];
        uint32_t boff[FR];
        float gr[FR][4];
#pragma unroll
        for (int j = 0; j < FR; ++j) {
            acc[j] = double4_t{0.0, 0.0, 0.0, 0.0};
            const int n = (g * FR + j) * 16 + lm;
            boff[j] = n < N ? (uint32_t)n * (uint32_t)K * 4u : kOOB;
        }
        // B values of one 16-k chunk: lane l holds k = 16*kc + 4*(l/16) + s, s = 0..3, of its column in each fragment
        // (A is read with the same k, so the products pair up whatever the order inside the chunk)
        auto load_b = [&](int kc, F4 (&b)[FR]) {
            const int k0 = kc * 16 + 4 * lk;
#pragma unroll
            for (int j = 0; j < FR; ++j)
                b[j] = buf_ld4<VEC>(rsrc, (boff[j] != kOOB && k0 < K) ? boff[j] + (uint32_t)k0 * 4u : kOOB, K - k0);
        };
        F4 ring[D][FR];
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < kchunks) load_b(d, ring[d]);
        // the relaxation entries of the epilogue do not depend on the products: requested now, used at the end
#pragma unroll
        for (int j = 0; j < FR; ++j) {
            const int n = (g * FR + j) * 16 + lm;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) gr[j][r4] = (st.grl && n < N) ? st.grl[(size_t)s_box[4 * r4 + lk] * N + n] : 1.f;
        }
        for (int kc0 = 0; kc0 < kchunks; kc0 += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int kc = kc0 + d;
                if (kc < kchunks) {
                    const float4 af = *reinterpret_cast<const float4*>(in + lm * si + kc * 16 + 4 * lk);
                    const double a[4] = {(double)af.x, (double)af.y, (double)af.z, (double)af.w};
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int j = 0; j < FR; ++j)
                            acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s], (double)ring[d][j].v[s], acc[j], 0, 0, 0);
                    if (kc + D < kchunks) load_b(kc + D, ring[d]);
                }
            }
        }
        // D: register r of lane l holds row 4*r + l/16, column l%16
#pragma unroll
        for (int j = 0; j < FR; ++j) {
            const int f = g * FR + j;
            if (f >= nfrag) continue;
            const int n = f * 16 + lm;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                double v = acc[j][r4];
                if (st.grl && n < N) v *= (double)relax_factor(v, gr[j][r4]);
                out[(4 * r4 + lk) * so + n] = (float)v;  // columns n >= N hold exact zeros (their weights read as 0)
            }
        }
    }
}

// The per-row sums over the block in LDS and the rows' bookkeeping.  A wave takes one task, i.e. the rows of +x and of
// -x of one neuron (same box: a neuron's constants are fetched once for both); a lane takes the columns lane,
// lane + 64, ...  What bounds this is the latency of the constants' fetches, so they are requested for U columns per
// lane at once, and for the first U columns BEFORE the product that makes the block (scan_fetch), so that the two
// latencies pass together.
template <int U>
struct ScanConsts {
    double cp[U], cn[U], X[U], kp[U], be[U];
    double xmax_self, xmax_a;        // per box: largest magnitudes of the block's own layer and of the next product's input
};
template <int U>
__device__ __forceinline__ void scan_fetch(const ChainStep& st, int b, int e0, ScanConsts<U>& k) {
    const int n = st.n;
    const size_t base = (size_t)b * n;
    k.xmax_self = (st.round_coef > 0.0 && st.xmax_self) ? st.xmax_self[b] : 0.0;
    k.xmax_a = (st.do_consts && st.xmax_a) ? st.xmax_a[b] : 0.0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int e = e0 + 64 * u;
        k.cp[u] = k.cn[u] = k.X[u] = k.kp[u] = k.be[u] = 0.0;
        if (e < n) {
            if (st.cpos) {
                k.cp[u] = st.cpos[base + e];
                k.cn[u] = st.cneg[base + e];
                k.X[u] = fmax(fabs(st.xlo[base + e]), fabs(st.xhi[base + e]));
            }
            if (st.do_consts) {
                if (st.kap) k.kp[u] = st.kap[base + e];
                if (st.beff) k.be[u] = st.beff[e];
            }
        }
    }
}
template <int U>
__device__ __forceinline__ void chain_scan(const ChainStep& st, const float* blk, int stride, ScanConsts<U>& k, int b,
                                           double* s_c, double* s_err, double* s_best, double coef_floor) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = st.n;
    const bool has_cand = st.cpos != nullptr;
    const bool dc = st.do_consts != 0;
    const int rows[2] = {wave, wave + CH_TASKS};
    const size_t base = (size_t)b * n;
    double cand[2] = {0, 0}, absx[2] = {0, 0}, cst[2] = {0, 0}, cstabs[2] = {0, 0}, s1[2] = {0, 0};
    for (int e0 = lane; e0 < n; e0 += 64 * U) {
        if (e0 != lane) scan_fetch<U>(st, b, e0, k);          // (the first U columns came in ahead of the product)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 64 * u;
            if (e < n) {
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    scan_term<float>(has_cand, dc, blk[rows[q] * stride + e], k.cp[u], k.cn[u], k.X[u], k.kp[u], k.be[u], cand[q],
                                     absx[q], cst[q], cstabs[q], s1[q]);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            cand[q] += __shfl_xor(cand[q], off, 64);
            absx[q] += __shfl_xor(absx[q], off, 64);
            cst[q] += __shfl_xor(cst[q], off, 64);
            cstabs[q] += __shfl_xor(cstabs[q], off, 64);
            s1[q] += __shfl_xor(s1[q], off, 64);
        }
    if (lane < 2) {
        const int q = lane, row = rows[q];
        const double t_cand = q ? cand[1] : cand[0], t_absx = q ? absx[1] : absx[0], t_cst = q ? cst[1] : cst[0],
                     t_cstabs = q ? cstabs[1] : cstabs[0], t_s1 = q ? s1[1] : s1[0];
        double c = s_c[row], err = s_err[row], best = s_best[row];
        const double floor_x = coef_floor * k.xmax_self;
        const double e1 = st.e1_a * k.xmax_a;
        scan_finish_math(n, st.round_coef, floor_x, has_cand, dc, e1, t_cand, t_absx, t_cst, t_cstabs, t_s1, c, err, best);
        s_c[row] = c; s_err[row] = err; s_best[row] = best;
    }
}

// the start layer's own matrix rows (+/-) over its predecessor, ReLU substitution applied: a wave takes one task, the
// matrix row is fetched once and stored as +row and as -row; U columns per lane are in flight together
template <int U>
__device__ __forceinline__ void chain_init(const ChainParams& p, const ChainStep& s0, float* cur, int cur_stride, int i, int b) {
    const int n = s0.n, n16 = (n + 15) & ~15;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t gb = (size_t)b * n;
    for (int e0 = lane; e0 < n16; e0 += 64 * U) {
        float w[U], gr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 64 * u;
            w[u] = 0.f; gr[u] = 1.f;
            if (e < n && i >= 0) {
                w[u] = p.w0[(size_t)i * n + e];
                if (s0.grl) gr[u] = s0.grl[gb + e];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + 64 * u;
            if (e >= n16) continue;
            float vp = w[u], vn = -w[u];
            if (s0.grl && w[u] != 0.f) {
                vp = (float)((double)vp * (double)relax_factor((double)vp, gr[u]));
                vn = (float)((double)vn * (double)relax_factor((double)vn, gr[u]));
            }
            cur[wave * cur_stride + e] = vp;
            cur[(wave + CH_TASKS) * cur_stride + e] = vn;
        }
    }
}

// one step: constants of the candidate requested, product, candidate.  PRE: request them before the product (short
// rows); for the long block over the input layer they would not fit beside the product's operands in registers.
template <int U, bool PRE>
__device__ __forceinline__ void chain_step(const ChainStep& st, const float* cur, int cur_stride, float* out, int out_stride,
                                           const int* s_box, double* s_c, double* s_err, double* s_best, double coef_floor) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = s_box[wave];
    ScanConsts<U> k;
    if (PRE) scan_fetch<U>(st, b, lane, k);
    const int per_wave = (((st.n + 15) >> 4) + CH_WAVES - 1) / CH_WAVES;      // column fragments per wave
    const bool vec = (st.K & 3) == 0;                                          // matrix rows start at multiples of 16 bytes
    if (per_wave <= 1) {
        if (vec) chain_cross<true, 1>(st, cur, cur_stride, out, out_stride, s_box);
        else chain_cross<false, 1>(st, cur, cur_stride, out, out_stride, s_box);
    } else if (PRE || per_wave == 2) {      // (PRE: rows of at most 256 columns, 16 fragments on 8 waves)
        if (vec) chain_cross<true, 2>(st, cur, cur_stride, out, out_stride, s_box);
        else chain_cross<false, 2>(st, cur, cur_stride, out, out_stride, s_box);
    } else if constexpr (!PRE) {
        if (vec) chain_cross<true, 4>(st, cur, cur_stride, out, out_stride, s_box);
        else chain_cross<false, 4>(st, cur, cur_stride, out, out_stride, s_box);
    }
    if (!PRE) scan_fetch<U>(st, b, lane, k);
    __syncthreads();
    chain_scan<U>(st, out, out_stride, k, b, s_c, s_err, s_best, coef_floor);
    __syncthreads();
}

}  // namespace

__global__ __launch_bounds__(CH_THREADS) void chain_kernel(const ChainParams p) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ double s_c[CH_ROWS], s_err[CH_ROWS], s_best[CH_ROWS];
    __shared__ int s_box[CH_ROWS], s_neuron[CH_ROWS];
    float* const hid[2] = {smem, smem + CH_ROWS * p.hid_stride};
    float* const last = smem + 2 * CH_ROWS * p.hid_stride;
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * CH_TASKS;
    if (tid < CH_ROWS) {
        const int t = t0 + (tid & 7);
        const bool valid = t < p.Rc;
        const uint32_t g = (uint32_t)(p.row0 + (valid ? t : p.Rc - 1));
        const uint32_t b = fast_div(g, p.div_n);
        s_box[tid] = (int)b;
        s_neuron[tid] = valid ? (int)(g - b * (uint32_t)p.n_start) : -1;
        const double bias = valid ? (double)p.bias0[g - b * (uint32_t)p.n_start] : 0.0;
        s_c[tid] = tid >= CH_TASKS ? -bias : bias;
        s_err[tid] = 0.0;
        s_best[tid] = INFINITY;
    }
    __syncthreads();

    // ---- step 0: the initial block and its candidate
    const ChainStep& s0 = p.steps[0];
    const bool only = p.nsteps == 1;
    float* cur = only ? last : hid[0];
    int cur_stride = only ? p.last_stride : p.hid_stride;
    {
        const int wave = tid >> 6, lane = tid & 63;
        const int b = s_box[wave], i = s_neuron[wave];
        if (s0.n <= 256) {
            ScanConsts<4> k;
            scan_fetch<4>(s0, b, lane, k);
            chain_init<4>(p, s0, cur, cur_stride, i, b);
            __syncthreads();
            chain_scan<4>(s0, cur, cur_stride, k, b, s_c, s_err, s_best, p.coef_floor);
        } else {
            ScanConsts<13> k;
            scan_fetch<13>(s0, b, lane, k);
            chain_init<13>(p, s0, cur, cur_stride, i, b);
            __syncthreads();
            chain_scan<13>(s0, cur, cur_stride, k, b, s_c, s_err, s_best, p.coef_floor);
        }
    }
    __syncthreads();

    // ---- the crossings, each followed by its candidate
    int which = 0;
    for (int s = 1; s < p.nsteps; ++s) {
        const ChainStep& st = p.steps[s];
        const bool to_last = s == p.nsteps - 1;
        float* out = to_last ? last : hid[which ^ 1];
        const int out_stride = to_last ? p.last_stride : p.hid_stride;
        if (st.n <= 128) chain_step<2, true>(st, cur, cur_stride, out, out_stride, s_box, s_c, s_err, s_best, p.coef_floor);
        else if (st.n <= 256) chain_step<4, true>(st, cur, cur_stride, out, out_stride, s_box, s_c, s_err, s_best, p.coef_floor);
        else chain_step<13, false>(st, cur, cur_stride, out, out_stride, s_box, s_c, s_err, s_best, p.coef_floor);
        cur = out; cur_stride = out_stride; which ^= 1;
    }

    // ---- store the bounds of the 8 neurons
    if (tid < CH_TASKS && s_neuron[tid] >= 0) {
        const long long g = (long long)p.row0 + t0 + tid;
        const double u = s_best[tid], l = -s_best[CH_TASKS + tid];
        if (!isfinite(u) || !isfinite(l)) *p.flag = 1;
        p.hi[g] = u;
        p.lo[g] = l;
        double x = fmax(fabs(u), fabs(l));
        if (!isfinite(x)) x = 0.0;
        // non-negative doubles order like their bit patterns
        atomicMax(reinterpret_cast<unsigned long long*>(p.xmax + s_box[tid]), (unsigned long long)__double_as_longlong(x));
        if (p.has_relu) {      // the ReLU layer that reads these bounds, neuron by neuron
            const double xr = relu_neuron(p.relu, g, l, u);
            atomicMax(reinterpret_cast<unsigned long long*>(p.relu.xmax + s_box[tid]), (unsigned long long)__double_as_longlong(xr));
        }
    }
}

size_t chain_lds_bytes(const ChainParams& p) {
    return sizeof(float) * (size_t)CH_ROWS * (2 * (size_t)p.hid_stride + (size_t)p.last_stride);
}

// Returns false when the kernel cannot be launched with the LDS it needs.
bool launch_chain(const ChainParams& p, hipStream_t s) {
    if (p.Rc <= 0) return true;
    const size_t lds = chain_lds_bytes(p);
    static size_t granted = 0;
    if (lds > granted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(chain_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        granted = lds;
    }
    hipLaunchKernelGGL(chain_kernel, dim3((p.Rc + CH_TASKS - 1) / CH_TASKS), dim3(CH_THREADS), lds, s, p);
    return true;
}

}  // namespace gp
