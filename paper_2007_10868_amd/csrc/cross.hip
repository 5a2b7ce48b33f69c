// HIP kernels of the DeepPoly back-substitution path for gfx950 (MI355X).
//
// Soundness scheme (the explicit-error-term alternative to the paper's interval coefficients,
// Section 4.1): coefficients are stored as ONE float32 value each; products of two float32
// values are exact in float64; sums are accumulated in float64 (MFMA f64); each new coefficient
// is rounded once to float32.  Every rounding is bounded and the bound, multiplied by the largest
// magnitude the neuron can take, is added to a per-row slack `err` that is part of every
// candidate bound.  All rows are upper-bound expressions (lower bounds are taken on -x).
// This file: crossing an affine layer (Algorithm 1 as an implicit GEMM), in several forms chosen by the width of the layer.
#include "device_common.hpp"

namespace gp {

// ------------------------------------------------------------------------------------------------
// Crossing an affine layer: per row a transposed convolution from the window in the layer's output
// to the window in its input (Algorithm 1), written as one implicit GEMM over all rows:
//   M = rows * out-window pixels, N = input channels, K = taps * output channels.
// A operand: gathered block values, with a pending ReLU substitution applied on the fly
//            (a * relax_factor, exact in float64).
// B operand: filter taps [tap][C_out][C_in].
// float64 MFMA 16x16x4; accumulators D[i][j]: lane l, register r holds i = 4*r + l/16, j = l%16.
// ------------------------------------------------------------------------------------------------
// Epilogue bookkeeping of one row: offset of the row's output pixel (window pixel (pa,pb)) in the packed relaxation
// of the input layer, [batch][Ho*Wo*Co], and in the addend block (-1 when the pixel lies outside the addend's window).
__device__ __forceinline__ void epilogue_row_info(const CrossParams& p, const RowInfo& ri, int r, int pa, int pb,
                                                  long long& ridx, long long& aoff) {
    const int N = p.Co;
    const int A = clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy) + pa;
    const int B = clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx) + pb;
    ridx = (long long)ri.b * ((long long)p.Ho * p.Wo * N) + (long long)(A * p.Wo + B) * N;
    aoff = -1;
    if (p.add.data) {
        const int ay = A - clampi(p.add.Sy * ri.ys - p.add.Py, 0, p.add.H - p.add.wy);
        const int ax = B - clampi(p.add.Sx * ri.xs - p.add.Px, 0, p.add.W - p.add.wx);
        if (ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx)
            aoff = ((long long)r * p.add.wy * p.add.wx + (long long)(ay * p.add.wx + ax)) * N;
    }
}

// LDS-tiled implicit GEMM on float64 MFMA (16x16x4).
//   Tile BM x BN per work-group of 4 waves, K step 16.  Both operand tiles are stored [row][k] with the
//   16 k-values of a row contiguous (row stride 18 doubles): a thread converts the 4 consecutive
//   channels it loaded (one 16-byte buffer load) and writes them with two 16-byte LDS stores; an MFMA
//   lane (row l%16, k-slot l/16) reads ITS 4 consecutive k-values back with two 16-byte LDS loads and
//   uses value j in MFMA step j, i.e. step j contracts the channel set {j, 4+j, 8+j, 12+j}.  A and B use
//   the same permutation, so every product pairs the right channels; only the summation order differs,
//   which the rounding slack covers for any order.
//   Vector instructions do not overlap float64 MFMAs on this chip (each costs 4-6 cycles of MFMA time; the chip's
//   float64 vector and matrix peaks are the same number), so everything outside the MFMAs is kept to a few
//   instructions per K step: 32-bit offsets into per-tile buffer resources, range-checked loads instead of masks,
//   tap geometry without divisions, per-row index arithmetic done once per row.
//   The K loop is software-pipelined (see the loop itself).  Layers with at most 32 input channels take
//   cross_direct_kernel below.
// Work decomposition: a work-group = (tile of BM rows, output pixel of the window, tile of BN input
// channels).  All rows of a work-group therefore produce the SAME window pixel, so the filter taps
// that can reach that pixel from inside the rows' windows are (nearly) the same for all of them: the taps
// that no row of the tile can use are skipped altogether (Algorithm 1 only visits pairs of a window entry
// and a tap; a gather over all taps of every output pixel would multiply many structural zeros, most of
// all for small windows and for strided layers).
// DENSE: the layer is a plain matrix (one tap, 1x1 windows): no tap geometry is kept, which leaves the registers for
// the software-pipelined K loop at 4 waves per SIMD without spilling.  The general 64x64 kernel is held to 4 waves per
// SIMD as well (a few values of the tap bookkeeping spill; measured: +3.4 % on the residual net against 3 waves).
// CT: storage type of the coefficient blocks (float; double for the float64 storage mode, which only this form and
// cross_pool_kernel serve: 32 bytes per 4 channels, no conversion, no rounding but the final one to float64).
template <int BM, int BN, bool VEC, bool DENSE, typename CT = float>
__global__ __launch_bounds__(256, (BM == 64 && BN == 64) ? 4 : 2) void cross_kernel(const CrossParams p) {
    constexpr bool A64 = std::is_same<CT, double>::value;
    constexpr uint32_t CS = sizeof(CT);
    constexpr int BK = 16;
    // float32 blocks are staged in LDS as they are and converted when a fragment is used: half the LDS traffic of a
    // float64 tile (the kernel's LDS reads and writes take a large share of the LDS bandwidth at full MFMA rate), the
    // same number of conversions per step for A, and the filter's conversions move from the staging to the use
    constexpr bool LDS32 = !A64;
    using LT = typename std::conditional<LDS32, float, double>::type;
    // elements per tile row: keeps 16-byte alignment, spreads banks (float: 80 B, 16 lanes x 16 B hit 64 distinct banks)
    constexpr int LDK = LDS32 ? 20 : 18;
    // the filter tile is staged as float64; the 16-byte forms read it from the weights' float64 copy, so that no
    // conversion of the filter operand is left in the K loop (measured: FC 9x500 +2.1 %, ResNet-34 +1.9 %); the
    // scalar-load forms and the general form of the float64 storage mode read the float32 weights and convert them
    // when they stage them
    constexpr bool BL32 = false;
    constexpr bool BG64 = VEC && (DENSE || !A64);     // the host launches these forms only with p.wt64 present
    using LTB = typename std::conditional<BL32, float, double>::type;
    constexpr int LDKB = BL32 ? 20 : 18;
    constexpr int WAVES_N = (BN >= 64 || BM < 64) ? 2 : 1;
    constexpr int WAVES_M = 4 / WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 16, TN = WTN / 16;
    constexpr int APT = (BM + 63) / 64;             // A rows per thread
    constexpr int BPT = (BN + 63) / 64;             // B columns per thread
    static_assert(TM >= 1 && TN >= 1, "tile");

    __shared__ __attribute__((aligned(16))) LT As[2][BM][LDK];
    __shared__ __attribute__((aligned(16))) LTB Bs[2][BN][LDKB];
    __shared__ unsigned long long s_tapmask;
    // per tile row, for the epilogue: where the row's output pixel sits in the relaxation array of the input layer and
    // in the addend block (-1: outside its window).  Worked out once per row by the thread that sets up the row's
    // loads; the 8 rows of an epilogue lane would otherwise each repeat the row's index arithmetic.
    __shared__ long long s_ridx[BM], s_aoff[BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int lk = lane >> 4, lm = lane & 15;
    const int opix = p.owy * p.owx;
    // Work-groups are dealt round-robin to the 8 XCDs, each with its own L2.  The logical tile order is
    // (row tile, pixel, channel tile) with the channel tile fastest, and XCD x takes the x-th contiguous
    // eighth of it: the work-groups that re-read the same rows of the block run on the same XCD at about the
    // same time, so the re-reads hit its L2 instead of HBM.
    const uint32_t total = (uint32_t)p.ntiles_n * (uint32_t)opix * (uint32_t)p.ntiles_m;
    const uint32_t per_xcd = (total + 7u) >> 3;
    const uint32_t logical = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;                              // whole work-group leaves before any barrier
    const uint32_t t2 = fast_div(logical, p.div_ntiles_n);
    const int nt = (int)(logical - t2 * (uint32_t)p.ntiles_n);
    const uint32_t rt = fast_div(t2, p.div_opix);
    const int pix = (int)(t2 - rt * (uint32_t)opix);           // window pixel of the tile (uniform)
    const int r_tile = (int)rt * BM;                           // first row of the tile
    const int pa = (int)fast_div((uint32_t)pix, p.div_owx), pb = pix - pa * p.owx;
    const int n0 = nt * BN;
    const int Ck = p.in.C, N = p.Co;
    const int taps = DENSE ? 1 : p.kh * p.kw;
    const int kchunks = (Ck + BK - 1) / BK;
    const uint32_t row_elems = (uint32_t)(p.in.wy * p.in.wx * Ck);

    // ---- buffer resources: A covers the rows of this tile only (32-bit offsets), B the layer's filter
    const int rows_here = min(BM, p.nrows - r_tile);
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(reinterpret_cast<const CT*>(p.in.data) + (size_t)r_tile * row_elems), 0, (int)((uint32_t)rows_here * row_elems * CS), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB =
        __builtin_amdgcn_make_buffer_rsrc((void*)p.wt, 0, (int)((uint32_t)taps * N * Ck * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB64 = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(BG64 ? (const void*)p.wt64 : (const void*)p.wt), 0, (int)((uint32_t)taps * N * Ck * (BG64 ? 8u : 4u)), 0x00020000);

    // ---- loader bookkeeping: thread -> (tile row ld_row (+64*i), channel quad q4)
    const int ld_row = tid >> 2, q4 = (tid & 3) * 4;
    // The rows of a tile are consecutive tasks, i.e. mostly the channels of ONE position of the start layer in one box:
    // then every row has the same window origins and can use the same taps, and the tap geometry is computed once, in
    // scalar registers (r_tile is uniform), instead of per thread in vector instructions that cost matrix time.
    const RowInfo u0 = row_info(p.rm, r_tile), u1 = row_info(p.rm, r_tile + rows_here - 1);
    const bool uni = !DENSE && p.rm.rowid == nullptr && u0.b == u1.b && u0.ys == u1.ys && u0.xs == u1.xs &&
                     (r_tile + rows_here <= p.rm.Rc || r_tile >= p.rm.Rc);
    const int u_oiy = clampi(p.in.Sy * u0.ys - p.in.Py, 0, p.in.H - p.in.wy);
    const int u_oix = clampi(p.in.Sx * u0.xs - p.in.Px, 0, p.in.W - p.in.wx);
    const int u_A = clampi(p.oSy * u0.ys - p.oPy, 0, p.Ho - p.owy) + pa, u_B = clampi(p.oSx * u0.xs - p.oPx, 0, p.Wo - p.owx) + pb;
    const uint32_t u_yy0 = (uint32_t)(u_A + p.ph), u_xx0 = (uint32_t)(u_B + p.pw);
    const int u_ydiv = (int)fast_div(u_yy0, p.div_sh), u_xdiv = (int)fast_div(u_xx0, p.div_sw);
    const int u_ymod = (int)(u_yy0 - (uint32_t)u_ydiv * (uint32_t)p.sh), u_xmod = (int)(u_xx0 - (uint32_t)u_xdiv * (uint32_t)p.sw);
    const int u_ty = p.in.tSy * u0.ys - p.in.tPy, u_tx = p.in.tSx * u0.xs - p.in.tPx;
    const int u_ylo = max(max(u_ty, u_oiy), 0), u_yhi = min(min(u_ty + p.in.tWy, u_oiy + p.in.wy), p.in.H);
    const int u_xlo = max(max(u_tx, u_oix), 0), u_xhi = min(min(u_tx + p.in.tWx, u_oix + p.in.wx), p.in.W);
    // tap t reaches this pixel from inside the common window?  poff = element offset of the window entry it reads
    auto tap_uniform = [&](int t, int& poff) -> bool {
        const int f = (int)fast_div((uint32_t)t, p.div_kw), g = t - f * p.kw;
        const int fdiv = (int)fast_div((uint32_t)f, p.div_sh), fmod = f - fdiv * p.sh;
        const int gdiv = (int)fast_div((uint32_t)g, p.div_sw), gmod = g - gdiv * p.sw;
        const int y = u_ydiv - fdiv, x = u_xdiv - gdiv;
        poff = ((y - u_oiy) * p.in.wx + (x - u_oix)) * Ck;
        return u_ymod == fmod && u_xmod == gmod && y >= u_ylo && y < u_yhi && x >= u_xlo && x < u_xhi;
    };
    uint32_t a_rowoff[APT];                 // byte offset of (row's block, channel q4) inside rsrcA
    int a_ydiv[APT], a_xdiv[APT], a_ymod[APT], a_xmod[APT], a_oiy[APT], a_oix[APT];
    uint32_t a_ty[APT], a_tx[APT];          // the row's exact window inside the stored one: first index | size << 16
    bool a_ok[APT];
#pragma unroll
    for (int i = 0; i < APT; ++i) {
        const int rl = ld_row + 64 * i;
        a_ok[i] = rl < rows_here;
        a_rowoff[i] = ((uint32_t)rl * row_elems + (uint32_t)q4) * CS;
        a_ydiv[i] = a_xdiv[i] = a_ymod[i] = a_xmod[i] = a_oiy[i] = a_oix[i] = 0;
        a_ty[i] = a_tx[i] = 0;
        if (uni) continue;
        const RowInfo ri = row_info(p.rm, r_tile + (a_ok[i] ? rl : 0));
        // window pixel (pa,pb) is pixel (A,B) of the input layer; tap (f,g) of the filter reads it from
        // layer-output pixel ((A + ph - f)/sh, (B + pw - g)/sw) when both divisions are exact
        const uint32_t yy0 = (uint32_t)(clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy) + pa + p.ph);
        const uint32_t xx0 = (uint32_t)(clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx) + pb + p.pw);
        const uint32_t yd = fast_div(yy0, p.div_sh), xd = fast_div(xx0, p.div_sw);
        a_ydiv[i] = (int)yd; a_ymod[i] = (int)(yy0 - yd * (uint32_t)p.sh);
        a_xdiv[i] = (int)xd; a_xmod[i] = (int)(xx0 - xd * (uint32_t)p.sw);
        a_oiy[i] = clampi(p.in.Sy * ri.ys - p.in.Py, 0, p.in.H - p.in.wy);
        a_oix[i] = clampi(p.in.Sx * ri.xs - p.in.Px, 0, p.in.W - p.in.wx);
        if constexpr (!DENSE) {
            // entries of the stored window outside the exact dependence window are structural zeros (border rows
            // keep a full-size window shifted inside the layer): taps that only reach those are not visited
            const int ty = p.in.tSy * ri.ys - p.in.tPy, tx = p.in.tSx * ri.xs - p.in.tPx;
            const int ylo = max(ty, a_oiy[i]), yhi = min(ty + p.in.tWy, a_oiy[i] + p.in.wy);
            const int xlo = max(tx, a_oix[i]), xhi = min(tx + p.in.tWx, a_oix[i] + p.in.wx);
            a_ty[i] = (uint32_t)(ylo - a_oiy[i]) | ((uint32_t)max(yhi - ylo, 0) << 16);
            a_tx[i] = (uint32_t)(xlo - a_oix[i]) | ((uint32_t)max(xhi - xlo, 0) << 16);
        }
        if ((tid & 3) == 0 && a_ok[i]) epilogue_row_info(p, ri, r_tile + rl, pa, pb, s_ridx[rl], s_aoff[rl]);
    }
    // per-thread byte offsets for the current tap: A row (kOOB when the tap misses the row's window), B column
    uint32_t a_voff[APT], b_voff[BPT];
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
        const int n = n0 + ld_row + 64 * i;
        const bool ok = (ld_row + 64 * i < BN) && n < N;
        b_voff[i] = ok ? ((uint32_t)n * (uint32_t)Ck + (uint32_t)q4) * 4u : kOOB;
    }
    // tap (f,g) written as f = fdiv*sh + fmod, g = gdiv*sw + gmod (all uniform); returns whether any of
    // this thread's rows uses the tap
    auto set_tap = [&](int t) -> bool {
        if constexpr (DENSE) {
#pragma unroll
            for (int i = 0; i < APT; ++i) a_voff[i] = a_ok[i] ? a_rowoff[i] : kOOB;
            return true;
        }
        const int f = (int)fast_div((uint32_t)t, p.div_kw), g = t - f * p.kw;
        const int fdiv = (int)fast_div((uint32_t)f, p.div_sh), fmod = f - fdiv * p.sh;
        const int gdiv = (int)fast_div((uint32_t)g, p.div_sw), gmod = g - gdiv * p.sw;
        bool any = false;
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            const int y = a_ydiv[i] - fdiv, x = a_xdiv[i] - gdiv;
            const int yi = y - a_oiy[i], xi = x - a_oix[i];
            const bool ok = a_ok[i] && a_ymod[i] == fmod && a_xmod[i] == gmod &&
                            (unsigned)y < (unsigned)p.in.H && (unsigned)x < (unsigned)p.in.W &&
                            (unsigned)(yi - (int)(a_ty[i] & 0xffffu)) < (a_ty[i] >> 16) &&
                            (unsigned)(xi - (int)(a_tx[i] & 0xffffu)) < (a_tx[i] >> 16);
            a_voff[i] = ok ? a_rowoff[i] + (uint32_t)(yi * p.in.wx + xi) * ((uint32_t)Ck * CS) : kOOB;
            any = any || ok;
        }
        return any;
    };

    // ---- which taps does this tile need at all?  (bit t of the mask; filters with more than 64 taps keep all)
    unsigned long long tapmask = ~0ull;
    uint32_t s_tapoff = 0;                       // uniform path: byte offset of the current tap's window entry (scalar)
    if (uni) {
#pragma unroll
        for (int i = 0; i < APT; ++i) a_voff[i] = a_ok[i] ? a_rowoff[i] : kOOB;
        if (taps <= 64) {
            unsigned long long m = 0;
            for (int t = 0; t < taps; ++t) {
                int poff;
                if (tap_uniform(t, poff)) m |= 1ull << t;
            }
            tapmask = m;
        }
    } else if (!DENSE && taps > 1 && taps <= 64) {
        unsigned long long mine = 0;
        for (int t = 0; t < taps; ++t)
            if (set_tap(t)) mine |= 1ull << t;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mine |= __shfl_xor(mine, off, 64);
        if (tid == 0) s_tapmask = 0;
        __syncthreads();
        if (lane == 0) atomicOr(&s_tapmask, mine);
        __syncthreads();
        tapmask = wave_uniform(s_tapmask);
    } else if (taps < 64) {
        tapmask = (1ull << taps) - 1;
    }
    // taps beyond 64 (huge filters) are all visited
    auto next_tap = [&](int t) -> int {          // first needed tap >= t, or taps (find-first-set, no loop over the bits)
        if (t >= 64 || t >= taps) return t;
        const unsigned long long m = tapmask >> t;
        return m ? min(t + (int)__builtin_ctzll(m), taps) : min(taps, 64);
    };
    // needed taps: the mask's bits below `taps`, and every tap from the 64th on
    const int n_taps = __builtin_popcountll(taps < 64 ? (tapmask & ((1ull << taps) - 1ull)) : tapmask) + max(taps - 64, 0);
    const int nIt = n_taps * kchunks;

    // the step the next loads are for moves on to tap t (uniform)
    auto enter_tap = [&](int t) {
        if (uni) {
            int poff;
            if (tap_uniform(t, poff)) {      // (filters with more than 64 taps visit all: a tap that misses reads nothing)
                s_tapoff = (uint32_t)poff * CS;
#pragma unroll
                for (int i = 0; i < APT; ++i) a_voff[i] = a_ok[i] ? a_rowoff[i] : kOOB;
            } else {
                s_tapoff = 0;
#pragma unroll
                for (int i = 0; i < APT; ++i) a_voff[i] = kOOB;
            }
        } else {
            set_tap(t);
        }
    };
    int ld_t = next_tap(0), ld_d0 = 0;
    if (ld_t < taps) enter_tap(ld_t);

    // global -> register staging holds raw float32 words only: nothing depends on the loads until the
    // MFMA loop of the current tile has been issued; conversion happens at the register -> LDS copy.
    // Per K step the loads cost no vector instruction: per-thread offsets are fixed within a tap and the
    // channel advance goes through the scalar offset operand of the buffer load.
    F4 a_raw[APT], b_raw[BPT];
    double a_raw64[A64 ? APT : 1][4];
    double b_raw64[BG64 ? BPT : 1][4];
    auto b_val = [&](int i, int j) -> double {
        if constexpr (BG64) return b_raw64[i][j];
        else return (double)b_raw[i].v[j];
    };
    auto a_val = [&](int i, int j) -> double {
        if constexpr (A64) return a_raw64[i][j];
        else return (double)a_raw[i].v[j];
    };
    // whole: the caller knows that the step is a whole 16-channel step of a dense layer and not its last one (no ragged
    // form, no move to another tap): the load then has no branch
    auto load_tiles = [&](auto whole_c) {
        constexpr bool WHOLE = DENSE && VEC && decltype(whole_c)::value;
        const int rem = Ck - ld_d0;                                 // channels left in this tap (uniform)
        const uint32_t soffA = s_tapoff + (uint32_t)ld_d0 * CS;
        const uint32_t soffB = ((uint32_t)ld_t * (uint32_t)N * (uint32_t)Ck + (uint32_t)ld_d0) * 4u;
        if (WHOLE || (VEC && rem >= BK)) {
#pragma unroll
            for (int i = 0; i < APT; ++i) {
                if constexpr (A64) {        // (kOOB + 16 is still beyond every range)
                    const uint4_t v0 = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soffA, 0);
                    const uint4_t v1 = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)(a_voff[i] + 16u), (int)soffA, 0);
                    a_raw64[i][0] = __hiloint2double((int)v0.y, (int)v0.x); a_raw64[i][1] = __hiloint2double((int)v0.w, (int)v0.z);
                    a_raw64[i][2] = __hiloint2double((int)v1.y, (int)v1.x); a_raw64[i][3] = __hiloint2double((int)v1.w, (int)v1.z);
                } else {
                    uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soffA, 0);
                    a_raw[i].v[0] = __uint_as_float(v.x); a_raw[i].v[1] = __uint_as_float(v.y);
                    a_raw[i].v[2] = __uint_as_float(v.z); a_raw[i].v[3] = __uint_as_float(v.w);
                }
            }
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                if constexpr (BG64) {       // byte offsets of the float64 copy are twice those of the float32 one
                    const uint32_t o = b_voff[i] == kOOB ? kOOB : 2u * b_voff[i];
                    const uint4_t v0 = __builtin_amdgcn_raw_buffer_load_b128(rsrcB64, (int)o, (int)(2u * soffB), 0);
                    const uint4_t v1 = __builtin_amdgcn_raw_buffer_load_b128(rsrcB64, (int)(o + 16u), (int)(2u * soffB), 0);
                    b_raw64[i][0] = __hiloint2double((int)v0.y, (int)v0.x); b_raw64[i][1] = __hiloint2double((int)v0.w, (int)v0.z);
                    b_raw64[i][2] = __hiloint2double((int)v1.y, (int)v1.x); b_raw64[i][3] = __hiloint2double((int)v1.w, (int)v1.z);
                } else {
                    uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, (int)b_voff[i], (int)soffB, 0);
                    b_raw[i].v[0] = __uint_as_float(v.x); b_raw[i].v[1] = __uint_as_float(v.y);
                    b_raw[i].v[2] = __uint_as_float(v.z); b_raw[i].v[3] = __uint_as_float(v.w);
                }
            }
        } else {                                                    // ragged last chunk of a tap, or unaligned channels
            const bool dok = q4 < rem;
#pragma unroll
            for (int i = 0; i < APT; ++i) {
                const uint32_t off = (dok && a_voff[i] != kOOB) ? a_voff[i] + soffA : kOOB;
                if constexpr (A64) buf_ld4_f64<VEC>(rsrcA, off, rem - q4, a_raw64[i]);
                else a_raw[i] = buf_ld4<VEC>(rsrcA, off, rem - q4);
            }
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                const bool ok = dok && b_voff[i] != kOOB;
                if constexpr (BG64) buf_ld4_f64<VEC>(rsrcB64, ok ? 2u * (b_voff[i] + soffB) : kOOB, rem - q4, b_raw64[i]);
                else b_raw[i] = buf_ld4<VEC>(rsrcB, ok ? b_voff[i] + soffB : kOOB, rem - q4);
            }
        }
        ld_d0 += BK;
        if constexpr (!WHOLE) {
            if (ld_d0 >= Ck) {                                      // next needed tap (uniform, once per kchunks steps)
                ld_d0 = 0;
                ld_t = next_tap(ld_t + 1);
                if (ld_t < taps) enter_tap(ld_t);
            }
        }
    };
    // LDS addresses of this thread's stores and MFMA operand loads (fixed; the buffer index is an immediate)
    LT* const a_st = &As[0][ld_row][q4];
    LTB* const b_st = &Bs[0][ld_row][q4];
    const LT* const a_ld = &As[0][wm * WTM + lm][4 * lk];
    const LTB* const b_ld = &Bs[0][wn * WTN + lm][4 * lk];
    // Last K step of a dense layer whose channel count is no multiple of 16 (e.g. 500 = 31*16 + 4): only tail_q of
    // the 4 channel quads exist.  Stored as usual they would sit in k-positions 0..4*tail_q-1, one in each of the 4
    // MFMA steps of the tile; stored transposed (channel j of quad q at k-position 4*j + q, for A and B alike) quad q
    // falls entirely into MFMA step q, and the steps >= tail_q, which would multiply zeros, are left out.
    const int tail_q = (DENSE && VEC && (Ck & 15)) ? ((Ck & 15) >> 2) : 0;
    auto store_tiles = [&](int buf, bool tail = false) {
        if (tail) {                                                 // uniform
            const int q = tid & 3;
            if (q < tail_q) {
#pragma unroll
                for (int i = 0; i < APT; ++i) {
                    if (BM % 64 == 0 || ld_row + 64 * i < BM) {    // (ld_row < 64)
                        LT* dst = &As[0][ld_row][0] + (buf * BM + 64 * i) * LDK + q;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if constexpr (LDS32) dst[4 * j] = a_raw[i].v[j];
                            else dst[4 * j] = a_val(i, j);
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < BPT; ++i) {
                    if (BN % 64 == 0 || ld_row + 64 * i < BN) {
                        LTB* dst = &Bs[0][ld_row][0] + (buf * BN + 64 * i) * LDKB + q;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if constexpr (BL32) dst[4 * j] = b_raw[i].v[j];
                            else dst[4 * j] = b_val(i, j);
                        }
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            if (BM % 64 == 0 || ld_row + 64 * i < BM) {    // (ld_row < 64)
                if constexpr (LDS32) {
                    *reinterpret_cast<float4*>(a_st + (buf * BM + 64 * i) * LDK) =
                        make_float4(a_raw[i].v[0], a_raw[i].v[1], a_raw[i].v[2], a_raw[i].v[3]);
                } else {
                    double2* dst = reinterpret_cast<double2*>(a_st + (buf * BM + 64 * i) * LDK);
                    dst[0] = make_double2(a_val(i, 0), a_val(i, 1));
                    dst[1] = make_double2(a_val(i, 2), a_val(i, 3));
                }
            }
        }
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            if (BN % 64 == 0 || ld_row + 64 * i < BN) {
                if constexpr (BL32) {
                    *reinterpret_cast<float4*>(b_st + (buf * BN + 64 * i) * LDKB) =
                        make_float4(b_raw[i].v[0], b_raw[i].v[1], b_raw[i].v[2], b_raw[i].v[3]);
                } else {
                    double2* dst = reinterpret_cast<double2*>(b_st + (buf * BN + 64 * i) * LDKB);
                    dst[0] = make_double2(b_val(i, 0), b_val(i, 1));
                    dst[1] = make_double2(b_val(i, 2), b_val(i, 3));
                }
            }
        }
    };

    double4_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};

    {
        // MFMA operand fragments of one K step: [half of the lane's 4 k-values][16-row tile], two sets so that the next
        // step's fragments are fetched from LDS while the MFMAs of the current step run
        double2 av[2][2][LDS32 ? 1 : TM], bv[2][2][BL32 ? 1 : TN];
        float4 av32[2][LDS32 ? TM : 1], bv32[2][BL32 ? TN : 1];
        auto read_frags = [&](auto set_c, int buf) {
            constexpr int set = decltype(set_c)::value;
            if constexpr (LDS32) {
    #pragma unroll
                for (int i = 0; i < TM; ++i)
                    av32[set][i] = *reinterpret_cast<const float4*>(a_ld + (buf * BM + i * 16) * LDK);
                if constexpr (BL32) {
    #pragma unroll
                    for (int j = 0; j < TN; ++j)
                        bv32[set][j] = *reinterpret_cast<const float4*>(b_ld + (buf * BN + j * 16) * LDKB);
                } else {
    #pragma unroll
                    for (int h = 0; h < 2; ++h)
    #pragma unroll
                        for (int j = 0; j < TN; ++j)
                            bv[set][h][j] = *reinterpret_cast<const double2*>(b_ld + (buf * BN + j * 16) * LDKB + 2 * h);
                }
                return;
            }
    #pragma unroll
            for (int h = 0; h < 2; ++h) {
    #pragma unroll
                for (int i = 0; i < TM; ++i)
                    av[set][h][i] = *reinterpret_cast<const double2*>(a_ld + (buf * BM + i * 16) * LDK + 2 * h);
    #pragma unroll
                for (int j = 0; j < TN; ++j)
                    bv[set][h][j] = *reinterpret_cast<const double2*>(b_ld + (buf * BN + j * 16) * LDKB + 2 * h);
            }
        };
        // quarter q of a step's 16 MFMAs: k-value q of each lane's four (halves h = q/2, component q%2)
        auto mfma_q = [&](auto set_c, auto q_c) {
            constexpr int set = decltype(set_c)::value, q = decltype(q_c)::value, h = q >> 1;
            if constexpr (LDS32) {
                double a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = (double)(q == 0 ? av32[set][i].x : q == 1 ? av32[set][i].y : q == 2 ? av32[set][i].z : av32[set][i].w);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if constexpr (BL32) b[j] = (double)(q == 0 ? bv32[set][j].x : q == 1 ? bv32[set][j].y : q == 2 ? bv32[set][j].z : bv32[set][j].w);
                    else b[j] = (q & 1) ? bv[set][h][j].y : bv[set][h][j].x;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
                return;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const double a = (q & 1) ? av[set][h][i].y : av[set][h][i].x;
                    const double b = (q & 1) ? bv[set][h][j].y : bv[set][h][j].x;
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[i][j], 0, 0, 0);
                }
        };
        using Q0 = std::integral_constant<int, 0>;
        using Q1 = std::integral_constant<int, 1>;
        using Q2 = std::integral_constant<int, 2>;
        using Q3 = std::integral_constant<int, 3>;
        // qlim: MFMA steps of the tile that hold data (4, or tail_q for the transposed last tile)
        auto mfma_head = [&](auto set_c, int qlim) {   // the MFMAs issued before the LDS write of the step (the split
            mfma_q(set_c, Q0{});                       // point makes no measurable difference: 4, 8 or 12 of the 16)
            if (qlim > 1) mfma_q(set_c, Q1{});
        };
        auto mfma_tail = [&](auto set_c, int qlim) {
            if (qlim > 2) mfma_q(set_c, Q2{});
            if (qlim > 3) mfma_q(set_c, Q3{});
        };
        using C0 = std::integral_constant<int, 0>;
        using C1 = std::integral_constant<int, 1>;
        const int last = nIt - 1;
        const int qlast = tail_q ? tail_q : 4;

        // Software pipeline over the K steps (tiles t = 0..nIt-1).  Per step, in program order: fetch the fragments
        // of tile t+1 from LDS; half of the MFMAs of tile t; convert and write tile t+2 into the LDS buffer whose
        // tile was turned into fragments one step ago; issue the global loads of tile t+3; the other MFMAs of tile
        // t; one barrier.  The LDS and global latencies of the coming tiles pass while the MFMAs of the current one
        // run, and nothing but the barrier stands between the MFMA phases of consecutive steps.
        if (nIt > 0) {
            load_tiles(std::false_type{});         // tile 0
            store_tiles(0, tail_q && last == 0);
            if (nIt > 1) load_tiles(std::false_type{});             // tile 1
            __syncthreads();
            read_frags(C0{}, 0);
            if (nIt > 1) store_tiles(1, tail_q && last == 1);
            if (nIt > 2) load_tiles(std::false_type{});             // tile 2
            __syncthreads();
            int t = 0;
            // STEADY: tiles t+2 .. t+4 exist and none of t+1 .. t+4 is the last one, so nothing in the pair of steps is
            // conditional (the compiled loop then has no branch between its MFMAs); the last pairs take the general form
            auto step_pair = [&](auto steady_c) {
                constexpr bool STEADY = decltype(steady_c)::value;
                read_frags(C1{}, 1);                       // tile t+1
                mfma_head(C0{}, 4);                        // tile t (never the last one here), first part
                __builtin_amdgcn_sched_barrier(0);
                if (STEADY || t + 2 < nIt) store_tiles(0, !STEADY && tail_q && t + 2 == last);   // tile t+2 (its loads were issued a step ago)
                if (STEADY || t + 3 < nIt) load_tiles(steady_c);   // tile t+3
                __builtin_amdgcn_sched_barrier(0);
                mfma_tail(C0{}, 4);                        // tile t, the rest
                __builtin_amdgcn_sched_barrier(0);         // keep the barrier (and its wait for the LDS traffic) behind the MFMAs
                __syncthreads();
                const int q1 = (!STEADY && t + 1 == last) ? qlast : 4;
                if (STEADY || t + 2 < nIt) read_frags(C0{}, 0);      // tile t+2
                mfma_head(C1{}, q1);                       // tile t+1
                __builtin_amdgcn_sched_barrier(0);
                if (STEADY || t + 3 < nIt) store_tiles(1, !STEADY && tail_q && t + 3 == last);   // tile t+3
                if (STEADY || t + 4 < nIt) load_tiles(steady_c);   // tile t+4
                __builtin_amdgcn_sched_barrier(0);
                mfma_tail(C1{}, q1);
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
            };
            for (; t + 5 < nIt; t += 2) step_pair(std::true_type{});
            for (; t + 2 <= nIt; t += 2) step_pair(std::false_type{});
            if (t < nIt) { mfma_head(C0{}, qlast); mfma_tail(C0{}, qlast); }   // odd number of tiles: the last one
        }
    }

    // ---- epilogue: (+ residual addend) (* ReLU substitution of the destination layer) -> one rounding to
    // float32 -> store.  D[i][j]: register r of lane l holds i = 4*r + l/16, j = l%16.
    __syncthreads();                                   // s_ridx, s_aoff (a tile without any tap has met no barrier yet)
    const bool has_add = p.add.data != nullptr;
    // A tile that no tap reaches (its pixel lies outside the exact dependence window of all of its rows) and that has no
    // addend holds zeros: written 16 bytes per thread where the alignment allows, with nothing to wait for.  (0 times a
    // relaxation factor is the same +0.)
    if (nIt == 0 && !has_add) {
        const int ncols = min(BN, N - n0);
        CT* const out0 = reinterpret_cast<CT*>(p.out) + ((size_t)r_tile * opix + pix) * N + n0;
        const size_t row_stride = (size_t)opix * N;
        if constexpr (!A64) {
            if ((N & 3) == 0 && (ncols & 3) == 0) {
                const int nq = ncols >> 2;
                for (int idx = tid; idx < rows_here * nq; idx += 256) {
                    const int rl = idx / nq, q = idx - rl * nq;
                    *reinterpret_cast<float4*>(out0 + (size_t)rl * row_stride + 4 * q) = make_float4(0.f, 0.f, 0.f, 0.f);
                }
                return;
            }
        }
        for (int idx = tid; idx < rows_here * ncols; idx += 256) {
            const int rl = idx / ncols, c = idx - rl * ncols;
            out0[(size_t)rl * row_stride + c] = (CT)0;
        }
        return;
    }
    // a dense layer's relaxation entry depends on the row's box only: when the whole tile lies in one box (within the
    // +x half and within the -x half rows are ordered by box) the lane's columns need one load each instead of one per row
    float g_same[TN];
    bool same_box = false;
    if constexpr (DENSE) {
        same_box = p.out_grl != nullptr && s_ridx[0] == s_ridx[rows_here - 1] &&
                   (r_tile + rows_here <= p.rm.Rc || r_tile >= p.rm.Rc);
        if (same_box) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * WTN + j * 16 + lm;
                g_same[j] = n < N ? p.out_grl[s_ridx[0] + n] : 0.f;
            }
        }
    }
    // uniform path: the pixel's place in the relaxation array and in the addend's window is the same for all rows
    const long long u_ridx = (long long)u0.b * ((long long)p.Ho * p.Wo * N) + (long long)(u_A * p.Wo + u_B) * N;
    long long u_aoff = -1;
    const long long u_astride = (long long)p.add.wy * p.add.wx * N;
    if (uni && has_add) {
        const int ay = u_A - clampi(p.add.Sy * u0.ys - p.add.Py, 0, p.add.H - p.add.wy);
        const int ax = u_B - clampi(p.add.Sx * u0.xs - p.add.Px, 0, p.add.W - p.add.wx);
        if (ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx) u_aoff = (long long)(ay * p.add.wx + ax) * N;
    }
    if (uni && p.out_grl) {
        same_box = true;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * WTN + j * 16 + lm;
            g_same[j] = n < N ? p.out_grl[u_ridx + n] : 0.f;
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int rl = wm * WTM + i * 16 + 4 * r4 + lk;              // register r4 of the lane is row 4*r4 + l/16
            const int r = r_tile + rl;
            if (r >= p.nrows) continue;
            const long long ridx = uni ? u_ridx : s_ridx[rl];
            const long long aoff = !has_add ? -1 : !uni ? s_aoff[rl] : u_aoff < 0 ? -1 : (long long)r * u_astride + u_aoff;
            const CT* add_src = aoff >= 0 ? reinterpret_cast<const CT*>(p.add.data) + aoff : nullptr;
            CT* out_row = reinterpret_cast<CT*>(p.out) + ((size_t)r * opix + pix) * N;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * WTN + j * 16 + lm;
                if (n >= N) continue;
                double v = acc[i][j][r4];
                if (add_src) v += (double)add_src[n];
                if (p.out_grl) v *= (double)relax_factor(v, same_box ? g_same[j] : p.out_grl[ridx + n]);
                out_row[n] = (CT)v;
            }
        }
    }
}

// Narrow layers (at most 32 input channels): the same implicit GEMM without LDS and without barriers.
//   With one wave across the N tile, an A value is needed by exactly one wave, in exactly the place the MFMA wants
//   it: lane l supplies A[row l%16][k l/16], so a lane that loads the 4 consecutive channels 4*(l/16)..+3 of row l%16
//   (one 16-byte buffer load; the four lanes of a row cover 64 contiguous bytes) holds its operand for the four MFMA
//   steps of a 16-channel K step, in the k-permutation described at cross_kernel.  The filter values are fetched the
//   same way (lane l: column l%16, the same 4 channels; they stay in the vector L1).  Every wave works on its own
//   16*TM rows and skips the taps that none of ITS rows can use; the next step's loads are issued before the MFMAs of
//   the current one and other waves' MFMAs cover what latency is left.
//   TN_ = 0 stands for layers with at most 4 input channels (the image).  A 16-column MFMA tile would be 13/16 padding
//   there; the 4x4x4 instruction (4 independent 4x4 blocks) keeps 16 rows per instruction with 4 columns.  Its operand
//   layout: lane l holds A[row l%16][k l/16] (as for 16x16x4), B[k l/16][column l%4] (the same B for every block), and
//   receives D[row 4*((l%16)/4) + l/16][column l%4].
template <int TM, int TN_, bool VEC>
__global__ __launch_bounds__(256, 2) void cross_direct_kernel(const CrossParams p) {
    constexpr bool SMALLN = (TN_ == 0);
    constexpr int TN = SMALLN ? 1 : TN_;
    constexpr int BK = 16;
    constexpr int BM = 64 * TM;                      // rows per work-group (4 waves of 16*TM rows)
    constexpr int BN = SMALLN ? 4 : 16 * TN;
    // epilogue bookkeeping per row (see cross_kernel); written and read by the same wave, so program order suffices
    __shared__ long long s_ridx[BM], s_aoff[BM];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lk = lane >> 4, lm = lane & 15;
    const int opix = p.owy * p.owx;
    const uint32_t total = (uint32_t)p.ntiles_n * (uint32_t)opix * (uint32_t)p.ntiles_m;
    const uint32_t per_xcd = (total + 7u) >> 3;
    const uint32_t logical = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);     // see cross_kernel
    if (logical >= total) return;
    const uint32_t t2 = fast_div(logical, p.div_ntiles_n);
    const int nt = (int)(logical - t2 * (uint32_t)p.ntiles_n);
    const uint32_t rt = fast_div(t2, p.div_opix);
    const int pix = (int)(t2 - rt * (uint32_t)opix);
    // Image layers: the filter (float64, 4 columns, the missing ones zero) is staged in LDS once per work-group.  With
    // 4 output columns a K step moves 1 KB of filter values per wave through the vector L1 next to 2 KB of block values,
    // and the L1 (64 B/clk) is what bounds these steps; from LDS the filter costs neither L1 traffic nor conversions.
    extern __shared__ __attribute__((aligned(16))) double s_w[];          // [tap][4][Ck + 2]
    const int ldw = p.in.C + 2;
    const bool lds_wt = SMALLN && p.lds_wt != 0;
    if (lds_wt) {
        const int Ck_ = p.in.C, cnt = p.kh * p.kw * 4 * Ck_;
        for (int idx = tid; idx < cnt; idx += 256) {
            const int c = idx % Ck_, tn = idx / Ck_, n = tn & 3, t = tn >> 2;
            s_w[tn * ldw + c] = n < p.Co ? p.wt64[((size_t)t * p.Co + n) * Ck_ + c] : 0.0;
        }
        __syncthreads();                                       // the only barrier; no wave has left yet
    }
    const int r_wave = (int)rt * BM + wave * 16 * TM;          // first row of this wave
    if (r_wave >= p.nrows) return;                             // no barrier anywhere below
    const int pa = (int)fast_div((uint32_t)pix, p.div_owx), pb = pix - pa * p.owx;
    const int n0 = nt * BN;
    const int Ck = p.in.C, N = p.Co;
    const int taps = p.kh * p.kw;
    const int kchunks = (Ck + BK - 1) / BK;
    const uint32_t row_elems = (uint32_t)(p.in.wy * p.in.wx * Ck);
    const int rows_here = min(16 * TM, p.nrows - r_wave);
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.in.data + (size_t)r_wave * row_elems), 0, (int)((uint32_t)rows_here * row_elems * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB =
        __builtin_amdgcn_make_buffer_rsrc((void*)p.wt, 0, (int)((uint32_t)taps * N * Ck * 4u), 0x00020000);

    const int q4 = 4 * lk;                       // this lane's channel quad inside a K step
    // The rows of a wave are consecutive tasks, i.e. mostly the channels of ONE position of the start layer in one box:
    // then every row has the same window origins and can use the same taps, and the whole tap geometry is computed
    // once, in scalar registers (r_wave is uniform), instead of per lane in vector instructions that cost matrix time.
    const RowInfo u0 = row_info(p.rm, r_wave), u1 = row_info(p.rm, r_wave + rows_here - 1);
    const bool uni = p.rm.rowid == nullptr && u0.b == u1.b && u0.ys == u1.ys && u0.xs == u1.xs &&
                     (r_wave + rows_here <= p.rm.Rc || r_wave >= p.rm.Rc);
    // uniform form of the geometry below (same formulas on the wave's common position)
    const int u_oiy = clampi(p.in.Sy * u0.ys - p.in.Py, 0, p.in.H - p.in.wy);
    const int u_oix = clampi(p.in.Sx * u0.xs - p.in.Px, 0, p.in.W - p.in.wx);
    const int u_A = clampi(p.oSy * u0.ys - p.oPy, 0, p.Ho - p.owy) + pa, u_B = clampi(p.oSx * u0.xs - p.oPx, 0, p.Wo - p.owx) + pb;
    const uint32_t u_yy0 = (uint32_t)(u_A + p.ph), u_xx0 = (uint32_t)(u_B + p.pw);
    const int u_ydiv = (int)fast_div(u_yy0, p.div_sh), u_xdiv = (int)fast_div(u_xx0, p.div_sw);
    const int u_ymod = (int)(u_yy0 - (uint32_t)u_ydiv * (uint32_t)p.sh), u_xmod = (int)(u_xx0 - (uint32_t)u_xdiv * (uint32_t)p.sw);
    const int u_ty = p.in.tSy * u0.ys - p.in.tPy, u_tx = p.in.tSx * u0.xs - p.in.tPx;
    const int u_ylo = max(max(u_ty, u_oiy), 0), u_yhi = min(min(u_ty + p.in.tWy, u_oiy + p.in.wy), p.in.H);
    const int u_xlo = max(max(u_tx, u_oix), 0), u_xhi = min(min(u_tx + p.in.tWx, u_oix + p.in.wx), p.in.W);
    // tap t reaches this pixel from inside the common window?  poff = element offset of the window entry it reads
    auto tap_uniform = [&](int t, int& poff) -> bool {
        const int f = (int)fast_div((uint32_t)t, p.div_kw), g = t - f * p.kw;
        const int fdiv = (int)fast_div((uint32_t)f, p.div_sh), fmod = f - fdiv * p.sh;
        const int gdiv = (int)fast_div((uint32_t)g, p.div_sw), gmod = g - gdiv * p.sw;
        const int y = u_ydiv - fdiv, x = u_xdiv - gdiv;
        poff = ((y - u_oiy) * p.in.wx + (x - u_oix)) * Ck;
        return u_ymod == fmod && u_xmod == gmod && y >= u_ylo && y < u_yhi && x >= u_xlo && x < u_xhi;
    };
    uint32_t a_rowoff[TM];
    int a_ydiv[TM], a_xdiv[TM], a_ymod[TM], a_xmod[TM], a_oiy[TM], a_oix[TM];
    uint32_t a_ty[TM], a_tx[TM];
    bool a_ok[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rl = i * 16 + lm;
        a_ok[i] = rl < rows_here;
        a_rowoff[i] = ((uint32_t)rl * row_elems + (uint32_t)q4) * 4u;
        a_ydiv[i] = a_xdiv[i] = a_ymod[i] = a_xmod[i] = a_oiy[i] = a_oix[i] = 0;
        a_ty[i] = a_tx[i] = 0;
        if (uni) continue;
        const RowInfo ri = row_info(p.rm, r_wave + (a_ok[i] ? rl : 0));
        const uint32_t yy0 = (uint32_t)(clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy) + pa + p.ph);
        const uint32_t xx0 = (uint32_t)(clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx) + pb + p.pw);
        const uint32_t yd = fast_div(yy0, p.div_sh), xd = fast_div(xx0, p.div_sw);
        a_ydiv[i] = (int)yd; a_ymod[i] = (int)(yy0 - yd * (uint32_t)p.sh);
        a_xdiv[i] = (int)xd; a_xmod[i] = (int)(xx0 - xd * (uint32_t)p.sw);
        a_oiy[i] = clampi(p.in.Sy * ri.ys - p.in.Py, 0, p.in.H - p.in.wy);
        a_oix[i] = clampi(p.in.Sx * ri.xs - p.in.Px, 0, p.in.W - p.in.wx);
        const int ty = p.in.tSy * ri.ys - p.in.tPy, tx = p.in.tSx * ri.xs - p.in.tPx;     // exact window, see cross_kernel
        const int ylo = max(ty, a_oiy[i]), yhi = min(ty + p.in.tWy, a_oiy[i] + p.in.wy);
        const int xlo = max(tx, a_oix[i]), xhi = min(tx + p.in.tWx, a_oix[i] + p.in.wx);
        a_ty[i] = (uint32_t)(ylo - a_oiy[i]) | ((uint32_t)max(yhi - ylo, 0) << 16);
        a_tx[i] = (uint32_t)(xlo - a_oix[i]) | ((uint32_t)max(xhi - xlo, 0) << 16);
        if (lk == 0 && a_ok[i])
            epilogue_row_info(p, ri, r_wave + rl, pa, pb, s_ridx[wave * 16 * TM + rl], s_aoff[wave * 16 * TM + rl]);
    }
    uint32_t a_voff[TM], b_voff[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = SMALLN ? n0 + (lm & 3) : n0 + j * 16 + lm;
        b_voff[j] = n < N ? ((uint32_t)n * (uint32_t)Ck + (uint32_t)q4) * 4u : kOOB;
    }
    auto set_tap = [&](int t) -> bool {
        const int f = (int)fast_div((uint32_t)t, p.div_kw), g = t - f * p.kw;
        const int fdiv = (int)fast_div((uint32_t)f, p.div_sh), fmod = f - fdiv * p.sh;
        const int gdiv = (int)fast_div((uint32_t)g, p.div_sw), gmod = g - gdiv * p.sw;
        bool any = false;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int y = a_ydiv[i] - fdiv, x = a_xdiv[i] - gdiv;
            const int yi = y - a_oiy[i], xi = x - a_oix[i];
            const bool ok = a_ok[i] && a_ymod[i] == fmod && a_xmod[i] == gmod &&
                            (unsigned)y < (unsigned)p.in.H && (unsigned)x < (unsigned)p.in.W &&
                            (unsigned)(yi - (int)(a_ty[i] & 0xffffu)) < (a_ty[i] >> 16) &&
                            (unsigned)(xi - (int)(a_tx[i] & 0xffffu)) < (a_tx[i] >> 16);
            a_voff[i] = ok ? a_rowoff[i] + (uint32_t)(yi * p.in.wx + xi) * (uint32_t)(Ck * 4) : kOOB;
            any = any || ok;
        }
        return any;
    };
    // taps some row of this wave can use (bit t; filters with more than 64 taps keep all)
    unsigned long long tapmask = ~0ull;
    uint32_t s_tapoff = 0;                       // uniform path: byte offset of the current tap's window entry (scalar)
    if (uni) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a_voff[i] = a_ok[i] ? a_rowoff[i] : kOOB;
        if (taps <= 64) {
            unsigned long long m = 0;
            for (int t = 0; t < taps; ++t) {
                int poff;
                if (tap_uniform(t, poff)) m |= 1ull << t;
            }
            tapmask = m;
        }
    } else if (taps <= 64) {
        unsigned long long mine = 0;
        for (int t = 0; t < taps; ++t)
            if (set_tap(t)) mine |= 1ull << t;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mine |= __shfl_xor(mine, off, 64);
        tapmask = wave_uniform(mine);
    }
    auto next_tap = [&](int t) -> int {          // see cross_kernel
        if (t >= 64 || t >= taps) return t;
        const unsigned long long m = tapmask >> t;
        return m ? min(t + (int)__builtin_ctzll(m), taps) : min(taps, 64);
    };
    // needed taps: the mask's bits below `taps`, and every tap from the 64th on
    const int n_taps = __builtin_popcountll(taps < 64 ? (tapmask & ((1ull << taps) - 1ull)) : tapmask) + max(taps - 64, 0);
    const int nIt = n_taps * kchunks;

    // the step the next loads are for moves on to tap t (uniform)
    auto enter_tap = [&](int t) {
        if (uni) {
            int poff;
            // (filters with more than 64 taps visit all of them: a tap that misses the window reads nothing)
            if (tap_uniform(t, poff)) {
                s_tapoff = (uint32_t)poff * 4u;
#pragma unroll
                for (int i = 0; i < TM; ++i) a_voff[i] = a_ok[i] ? a_rowoff[i] : kOOB;
            } else {
                s_tapoff = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i) a_voff[i] = kOOB;
            }
        } else {
            set_tap(t);
        }
    };
    int ld_t = next_tap(0), ld_d0 = 0;
    if (ld_t < taps) enter_tap(ld_t);
    // the epilogue's relaxation entries on the uniform path, requested now so that their latency passes under the K loop
    const long long u_ridx = (long long)u0.b * ((long long)p.Ho * p.Wo * N) + (long long)(u_A * p.Wo + u_B) * N;
    float g_uni[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = SMALLN ? n0 + (lm & 3) : n0 + j * 16 + lm;
        g_uni[j] = (uni && p.out_grl && n < N) ? p.out_grl[u_ridx + n] : 0.f;
    }
    F4 a_raw[TM], b_raw[TN];
    auto load_step = [&]() {
        const int rem = Ck - ld_d0;
        const uint32_t soffA = s_tapoff + (uint32_t)ld_d0 * 4u;
        const uint32_t soffB = ((uint32_t)ld_t * (uint32_t)N * (uint32_t)Ck + (uint32_t)ld_d0) * 4u;
        if (VEC && rem >= BK) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soffA, 0);
                a_raw[i].v[0] = __uint_as_float(v.x); a_raw[i].v[1] = __uint_as_float(v.y);
                a_raw[i].v[2] = __uint_as_float(v.z); a_raw[i].v[3] = __uint_as_float(v.w);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, (int)b_voff[j], (int)soffB, 0);
                b_raw[j].v[0] = __uint_as_float(v.x); b_raw[j].v[1] = __uint_as_float(v.y);
                b_raw[j].v[2] = __uint_as_float(v.z); b_raw[j].v[3] = __uint_as_float(v.w);
            }
        } else {
            const bool dok = q4 < rem;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a_raw[i] = buf_ld4<VEC>(rsrcA, (dok && a_voff[i] != kOOB) ? a_voff[i] + soffA : kOOB, rem - q4);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b_raw[j] = buf_ld4<VEC>(rsrcB, (dok && b_voff[j] != kOOB) ? b_voff[j] + soffB : kOOB, rem - q4);
        }
        ld_d0 += BK;
        if (ld_d0 >= Ck) {
            ld_d0 = 0;
            ld_t = next_tap(ld_t + 1);
            if (ld_t < taps) enter_tap(ld_t);
        }
    };

    double4_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};

    auto convert = [&](double (&av)[TM][4], double (&bv)[TN][4]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int k = 0; k < 4; ++k) av[i][k] = (double)a_raw[i].v[k];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k) bv[j][k] = (double)b_raw[j].v[k];
    };
    auto mfmas = [&](const double (&av)[TM][4], const double (&bv)[TN][4]) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (SMALLN)
                        acc[i][0][0] = __builtin_amdgcn_mfma_f64_4x4x4f64(av[i][k], bv[0][k], acc[i][0][0], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[i][k], bv[j][k], acc[i][j], 0, 0, 0);
                }
    };
    if (VEC && (Ck & (BK - 1)) == 0) {
        // Whole K steps only.  One step is ONE basic block - convert the step's raw values, issue the next step's loads,
        // then the MFMAs - with the order pinned: the loads stay in flight while the MFMAs run.  (With branches between
        // them the compiler moves the MFMAs ahead of the loads and every step waits for its own loads.)  The loads are
        // unconditional: behind the last step they re-read the current rows (A) and run off the filter's range (B, zeros).
        auto issue = [&]() {
            const uint32_t soffA = s_tapoff + (uint32_t)ld_d0 * 4u;
            const uint32_t soffB = ((uint32_t)ld_t * (uint32_t)N * (uint32_t)Ck + (uint32_t)ld_d0) * 4u;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soffA, 0);
                a_raw[i].v[0] = __uint_as_float(v.x); a_raw[i].v[1] = __uint_as_float(v.y);
                a_raw[i].v[2] = __uint_as_float(v.z); a_raw[i].v[3] = __uint_as_float(v.w);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, (int)b_voff[j], (int)soffB, 0);
                b_raw[j].v[0] = __uint_as_float(v.x); b_raw[j].v[1] = __uint_as_float(v.y);
                b_raw[j].v[2] = __uint_as_float(v.z); b_raw[j].v[3] = __uint_as_float(v.w);
            }
        };
        auto advance = [&]() {                      // the step the next loads are for (uniform)
            ld_d0 += BK;
            if (ld_d0 >= Ck) {
                ld_d0 = 0;
                ld_t = next_tap(ld_t + 1);
                if (ld_t < taps) enter_tap(ld_t);
            }
        };
        if (lds_wt) {
            // block values as above (the filter loads of issue() are dead here and drop out); the filter fragment of
            // the NEXT step is fetched from LDS while the MFMAs of this one run
            auto issue_a = [&]() {
                const uint32_t soffA = s_tapoff + (uint32_t)ld_d0 * 4u;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soffA, 0);
                    a_raw[i].v[0] = __uint_as_float(v.x); a_raw[i].v[1] = __uint_as_float(v.y);
                    a_raw[i].v[2] = __uint_as_float(v.z); a_raw[i].v[3] = __uint_as_float(v.w);
                }
            };
            const double* const w_lane = s_w + (lm & 3) * ldw + q4;
            auto filter_frag = [&](int t, int d0, double (&b)[4]) {
                const int tt = min(t, taps - 1);                // behind the last step: any valid address
                const double2* src = reinterpret_cast<const double2*>(w_lane + tt * 4 * ldw + d0);
                const double2 x = src[0], y = src[1];
                b[0] = x.x; b[1] = x.y; b[2] = y.x; b[3] = y.y;
            };
            double bcur[4] = {0.0, 0.0, 0.0, 0.0}, bnext[4];
            if (nIt > 0) { filter_frag(ld_t, ld_d0, bcur); issue_a(); advance(); }
            for (int it = 0; it < nIt; ++it) {
                double av[TM][4], bv[TN][4];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int k = 0; k < 4; ++k) av[i][k] = (double)a_raw[i].v[k];
#pragma unroll
                for (int k = 0; k < 4; ++k) bv[0][k] = bcur[k];
                __builtin_amdgcn_sched_barrier(0);
                issue_a();
                filter_frag(ld_t, ld_d0, bnext);
                __builtin_amdgcn_sched_barrier(0);
                mfmas(av, bv);
                __builtin_amdgcn_sched_barrier(0);
                advance();
#pragma unroll
                for (int k = 0; k < 4; ++k) bcur[k] = bnext[k];
            }
        } else {
            if (nIt > 0) { issue(); advance(); }
            for (int it = 0; it < nIt; ++it) {
                double av[TM][4], bv[TN][4];
                convert(av, bv);
                __builtin_amdgcn_sched_barrier(0);
                issue();
                __builtin_amdgcn_sched_barrier(0);
                mfmas(av, bv);
                __builtin_amdgcn_sched_barrier(0);
                advance();
            }
        }
    } else {
        if (nIt > 0) load_step();
        for (int it = 0; it < nIt; ++it) {
            double av[TM][4], bv[TN][4];
            convert(av, bv);
            if (it + 1 < nIt) load_step();
            mfmas(av, bv);
        }
    }

    // ---- epilogue, as in cross_kernel; on the uniform path the pixel's place in the relaxation array and in the
    // addend's window is the same for all rows (the addend block itself is per row)
    const bool has_add = p.add.data != nullptr;
    long long u_aoff = -1;
    const long long u_astride = (long long)p.add.wy * p.add.wx * N;
    if (uni && has_add) {
        const int ay = u_A - clampi(p.add.Sy * u0.ys - p.add.Py, 0, p.add.H - p.add.wy);
        const int ax = u_B - clampi(p.add.Sx * u0.xs - p.add.Px, 0, p.add.W - p.add.wx);
        if (ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx) u_aoff = (long long)(ay * p.add.wx + ax) * N;
    }
    // uniform path: the lane's columns have ONE relaxation entry each, whatever the row (g_uni, requested before the K
    // loop): the two multipliers a coefficient can take (upper slope for a >= 0, lower slope 0 or 1 for a < 0) are
    // formed once per column
    double g_pos[TN], g_neg[TN];
    if (uni && p.out_grl) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            g_pos[j] = (double)fabsf(g_uni[j]);
            g_neg[j] = signbit(g_uni[j]) ? 0.0 : 1.0;
        }
    }
    // stores through a buffer resource over the wave's rows: 32-bit offsets
    const uint32_t out_row_bytes = (uint32_t)opix * (uint32_t)N * 4u;
    const __amdgpu_buffer_rsrc_t rsrcO = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.out + (size_t)r_wave * opix * N), 0, (int)((uint32_t)rows_here * out_row_bytes), 0x00020000);
    // A tile that no tap reaches (its pixel lies outside the exact dependence window of all of the wave's rows) and that
    // has no addend holds zeros: they are written 16 bytes per lane, with nothing to wait for.  (0 times a relaxation
    // factor is the same +0.)
    if (nIt == 0 && !has_add) {
        const int ncols = min(BN, N - n0);
        if ((N & 3) == 0 && (ncols & 3) == 0) {
            const int nq = ncols >> 2;
            for (int idx = lane; idx < rows_here * nq; idx += 64) {
                const int rl = idx / nq, q = idx - rl * nq;
                __builtin_amdgcn_raw_buffer_store_b128(uint4_t{0u, 0u, 0u, 0u}, rsrcO,
                    (int)((uint32_t)rl * out_row_bytes + ((uint32_t)pix * (uint32_t)N + (uint32_t)(n0 + 4 * q)) * 4u), 0, 0);
            }
        } else {
            for (int idx = lane; idx < rows_here * ncols; idx += 64) {
                const int rl = idx / ncols, c = idx - rl * ncols;
                __builtin_amdgcn_raw_buffer_store_b32(0u, rsrcO,
                    (int)((uint32_t)rl * out_row_bytes + ((uint32_t)pix * (uint32_t)N + (uint32_t)(n0 + c)) * 4u), 0, 0);
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r4 = 0; r4 < (SMALLN ? 1 : 4); ++r4) {
            // 16x16x4: register r4 of the lane is row 4*r4 + l/16; 4x4x4: the lane's one value is row 4*((l%16)/4) + l/16
            const int rl = i * 16 + (SMALLN ? 4 * (lm >> 2) : 4 * r4) + lk;
            const int r = r_wave + rl;
            if (r >= p.nrows) continue;
            const long long ridx = uni ? u_ridx : s_ridx[wave * 16 * TM + rl];
            const long long aoff = !has_add ? -1 : !uni ? s_aoff[wave * 16 * TM + rl] : u_aoff < 0 ? -1 : (long long)r * u_astride + u_aoff;
            const float* add_src = aoff >= 0 ? p.add.data + aoff : nullptr;
            const uint32_t out_off = (uint32_t)rl * out_row_bytes + (uint32_t)pix * (uint32_t)N * 4u;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = SMALLN ? n0 + (lm & 3) : n0 + j * 16 + lm;
                if (n >= N) continue;
                double v = acc[i][j][r4];
                if (add_src) v += (double)add_src[n];
                if (p.out_grl) {
                    if (uni) v *= (v >= 0.0 ? g_pos[j] : g_neg[j]);
                    else v *= (double)relax_factor(v, p.out_grl[ridx + n]);
                }
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint((float)v), rsrcO, (int)(out_off + (uint32_t)n * 4u), 0, 0);
            }
        }
    }
}

template <int TM, int TN>
static void launch_cross_direct(const CrossParams& p0, hipStream_t s) {
    constexpr int BM = 64 * TM, BN = TN == 0 ? 4 : 16 * TN;
    CrossParams p = p0;
    p.ntiles_m = (p.nrows + BM - 1) / BM;
    p.ntiles_n = (p.Co + BN - 1) / BN;
    p.div_ntiles_n = make_fastdiv((uint32_t)p.ntiles_n);
    p.div_opix = make_fastdiv((uint32_t)(p.owy * p.owx));
    const long long total = (long long)p.ntiles_m * p.ntiles_n * p.owy * p.owx;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    // image layers: filter in LDS when its float64 copy exists, the K steps are whole and it fits beside 8 work-groups
    const size_t w_bytes = (size_t)p.kh * p.kw * 4 * (p.in.C + 2) * sizeof(double);
    p.lds_wt = (TN == 0 && p.wt64 && (p.in.C & 15) == 0 && w_bytes <= 24576) ? 1 : 0;
    const size_t lds = p.lds_wt ? w_bytes : 0;
    if ((p.in.C & 3) == 0) hipLaunchKernelGGL((cross_direct_kernel<TM, TN, true>), dim3(blocks), dim3(256), lds, s, p);
    else hipLaunchKernelGGL((cross_direct_kernel<TM, TN, false>), dim3(blocks), dim3(256), lds, s, p);
}

// Layers with at most 4 input channels (the image): no matrix instruction.  An output pixel of such a step has N <= 4
// values and, behind a strided layer, K = (taps that reach it) * channels of a few dozen: a work-group per pixel
// would spend its time on bookkeeping.  Here ONE LANE computes one (row, output pixel): it walks the taps that can
// reach its pixel and the channels under each tap and accumulates N float64 sums with fused multiply-adds (whose
// peak on this chip equals the float64 MFMA peak).  Lanes are grouped by the pixel's PARITY CLASS, i.e. by
// ((A + ph) mod sh, (B + pw) mod sw) of its absolute position (A, B): within a class every lane uses the same taps
// f = cy + t*sh, g = cx + u*sw, so tap and channel loops are uniform and the (float64) filter values come through
// scalar loads.
// A work-group owns R consecutive rows.  It copies their blocks into LDS once, converted to float64 (a block value is
// used by every output pixel a tap links it to, ceil(kh/sh)*ceil(kw/sw) of them: read per use from global memory, the
// lanes of a wave fetched 16 bytes each out of 64 different 64-byte segments and the vector L1 set the pace).  In LDS a
// block pixel is padded by 2 doubles, so that lanes on neighbouring pixels hit different banks.  A wave then takes a
// (class, group of 64*NIT items) unit: per tap and 4-channel step the filter values are loaded once and used for the
// NIT items of every lane.  A tap that misses an item's window reads a pixel of zeros instead (adding 0*w leaves a
// sum as it is), so the loops have no divergent branch.  Per (item, column) the products are added in the order tap
// row, tap column, channel, whatever R and NIT are.
// grid: x over groups of R rows.
constexpr int IMG_NIT = 4;
constexpr int IMG_RMAX = 64;            // rows per work-group at most (their geometry sits in a table in LDS)
template <int NN, bool VEC>      // NN: input channels of the layer (columns of the step)
__global__ __launch_bounds__(256) void cross_image_kernel(const CrossParams p, int R, int pstride, int ngroups) {
    constexpr int NIT = IMG_NIT;
    extern __shared__ __attribute__((aligned(16))) double s_blk[];       // [R * window pixels + 1][pstride]
    // what an item needs of its row, worked out once per row: {box, oy, ox, (oy+ph) mod sh}, {(ox+pw) mod sw, oiy, oix,
    // 0}, {exact window inside the stored one: first row | rows << 16, first column | columns << 16, 0, 0}
    __shared__ int4 s_row[IMG_RMAX][3];
    constexpr int N = NN;
    const int Ck = p.in.C;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int npix_in = p.in.wy * p.in.wx, row_elems = npix_in * Ck;
    const int r0 = blockIdx.x * R, rows_here = min(R, p.nrows - r0);
    const int ppc = p.cls_ny * p.cls_nx;
    const int zero_pix = R * npix_in;                                    // the pixel of zeros
    if (tid < rows_here) {
        const RowInfo ri = row_info(p.rm, r0 + tid);
        const int oy = clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy), ox = clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx);
        const uint32_t my = (uint32_t)(oy + p.ph), mx = (uint32_t)(ox + p.pw);
        const int oiy = clampi(p.in.Sy * ri.ys - p.in.Py, 0, p.in.H - p.in.wy), oix = clampi(p.in.Sx * ri.xs - p.in.Px, 0, p.in.W - p.in.wx);
        // the part of the row's stored window that lies in its exact dependence window (see cross_kernel)
        const int ty = p.in.tSy * ri.ys - p.in.tPy, tx = p.in.tSx * ri.xs - p.in.tPx;
        const int ylo = max(ty, oiy), yhi = min(ty + p.in.tWy, oiy + p.in.wy);
        const int xlo = max(tx, oix), xhi = min(tx + p.in.tWx, oix + p.in.wx);
        s_row[tid][0] = make_int4(ri.b, oy, ox, (int)(my - fast_div(my, p.div_sh) * (uint32_t)p.sh));
        s_row[tid][1] = make_int4((int)(mx - fast_div(mx, p.div_sw) * (uint32_t)p.sw), oiy, oix, 0);
        s_row[tid][2] = make_int4((int)((uint32_t)(ylo - oiy) | ((uint32_t)max(yhi - ylo, 0) << 16)),
                                  (int)((uint32_t)(xlo - oix) | ((uint32_t)max(xhi - xlo, 0) << 16)), 0, 0);
    }
    // ---- the rows' blocks -> LDS (float64)
    {
        const float* src = p.in.data + (size_t)r0 * row_elems;
        const int total = rows_here * row_elems;
        if (VEC) {
            for (int e = tid * 4; e < total; e += 1024) {
                const float4 v = *reinterpret_cast<const float4*>(src + e);
                const int pix = (int)fast_div((uint32_t)e, p.div_ntiles_n);      // div_ntiles_n: the launcher's divider by Ck
                double* dst = s_blk + pix * pstride + (e - pix * Ck);
                reinterpret_cast<double2*>(dst)[0] = make_double2((double)v.x, (double)v.y);
                reinterpret_cast<double2*>(dst)[1] = make_double2((double)v.z, (double)v.w);
            }
        } else {
            for (int e = tid; e < total; e += 256) {
                const int pix = (int)fast_div((uint32_t)e, p.div_ntiles_n);
                s_blk[pix * pstride + (e - pix * Ck)] = (double)src[e];
            }
        }
        for (int c = tid; c < pstride; c += 256) s_blk[zero_pix * pstride + c] = 0.0;
    }
    __syncthreads();
    const int ncls = p.sh * p.sw;
    for (int unit = wave; unit < ncls * ngroups; unit += 4) {              // uniform per wave
        const int cls = unit % ncls, grp = unit / ncls;
        const int cy = (int)fast_div((uint32_t)cls, p.div_sw), cx = cls - cy * p.sw;
        // ---- the lane's items
        int base[NIT], yrel[NIT], xrel[NIT];             // LDS pixel index of the row's block; tap (0,0) reads window entry (yrel, xrel)
        uint32_t yrng[NIT], xrng[NIT];                   // exact dependence window inside the stored one: first | size << 16
        int item_rho[NIT], item_pix[NIT];                // row within the group; window pixel pa << 16 | pb (-1: no item)
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int idx = (grp * NIT + i) * 64 + lane;
            item_pix[i] = -1;
            base[i] = 0; yrel[i] = xrel[i] = 0; yrng[i] = xrng[i] = 0; item_rho[i] = 0;
            if (idx >= rows_here * ppc) continue;
            const uint32_t rho = fast_div((uint32_t)idx, p.div_cls);
            const uint32_t k = (uint32_t)idx - rho * (uint32_t)ppc;
            const uint32_t ky = fast_div(k, p.div_cls_nx), kx = k - ky * (uint32_t)p.cls_nx;
            const int4 g0 = s_row[rho][0], g1 = s_row[rho][1], g2 = s_row[rho][2];
            // first window pixel of the class: pa = cy - (oy + ph) (mod sh)
            int pa = cy - g0.w, pb = cx - g1.x;
            pa += (pa < 0 ? p.sh : 0) + (int)ky * p.sh;
            pb += (pb < 0 ? p.sw : 0) + (int)kx * p.sw;
            if (pa >= p.owy || pb >= p.owx) continue;
            const int A = g0.y + pa, B = g0.z + pb;
            // tap (f, g) = (cy + t*sh, cx + u*sw) reads layer-output pixel (y0 - t, x0 - u)
            const int y0 = (int)fast_div((uint32_t)(A + p.ph - cy), p.div_sh), x0 = (int)fast_div((uint32_t)(B + p.pw - cx), p.div_sw);
            base[i] = (int)rho * npix_in;
            yrel[i] = y0 - g1.y; xrel[i] = x0 - g1.z;
            yrng[i] = (uint32_t)g2.x; xrng[i] = (uint32_t)g2.y;
            item_rho[i] = (int)rho; item_pix[i] = (pa << 16) | pb;
        }
        double acc[NIT][N];
#pragma unroll
        for (int i = 0; i < NIT; ++i)
#pragma unroll
            for (int n = 0; n < N; ++n) acc[i][n] = 0.0;
        for (int t = 0, f = cy; f < p.kh; ++t, f += p.sh) {                  // uniform loops
            for (int u = 0, g = cx; g < p.kw; ++u, g += p.sw) {
                const double* a[NIT];
#pragma unroll
                for (int i = 0; i < NIT; ++i) {
                    const int y = yrel[i] - t, x = xrel[i] - u;
                    const bool ok = item_pix[i] >= 0 && (unsigned)(y - (int)(yrng[i] & 0xffffu)) < (yrng[i] >> 16) &&
                                    (unsigned)(x - (int)(xrng[i] & 0xffffu)) < (xrng[i] >> 16);
                    a[i] = s_blk + (ok ? base[i] + y * p.in.wx + x : zero_pix) * pstride;
                }
                const double* w = p.wt64 + (size_t)(f * p.kw + g) * N * Ck;     // [n][c], uniform
                if (VEC) {
                    for (int c = 0; c < Ck; c += 4) {
                        // the block values of all items first, so that their LDS latencies pass together
                        double av[NIT][4];
#pragma unroll
                        for (int i = 0; i < NIT; ++i) {
                            const double2 a0 = reinterpret_cast<const double2*>(a[i] + c)[0];
                            const double2 a1 = reinterpret_cast<const double2*>(a[i] + c)[1];
                            av[i][0] = a0.x; av[i][1] = a0.y; av[i][2] = a1.x; av[i][3] = a1.y;
                        }
                        double wv[N][4];
#pragma unroll
                        for (int n = 0; n < N; ++n)
#pragma unroll
                            for (int j = 0; j < 4; ++j) wv[n][j] = w[n * Ck + c + j];
#pragma unroll
                        for (int i = 0; i < NIT; ++i)
#pragma unroll
                            for (int n = 0; n < N; ++n)
#pragma unroll
                                for (int j = 0; j < 4; ++j) acc[i][n] = fma(av[i][j], wv[n][j], acc[i][n]);
                    }
                } else {
                    for (int c = 0; c < Ck; ++c) {
                        double av[NIT];
#pragma unroll
                        for (int i = 0; i < NIT; ++i) av[i] = a[i][c];
#pragma unroll
                        for (int i = 0; i < NIT; ++i)
#pragma unroll
                            for (int n = 0; n < N; ++n) acc[i][n] = fma(av[i], w[n * Ck + c], acc[i][n]);
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            if (item_pix[i] < 0) continue;
            const int r = r0 + item_rho[i];
            const int pa = item_pix[i] >> 16, pb = item_pix[i] & 0xffff;
            const int4 g0 = s_row[item_rho[i]][0];
            // place of the pixel in the packed relaxation of the input layer, [box][Ho*Wo*Co]
            long long ridx = (long long)g0.x * ((long long)p.Ho * p.Wo * N) + (long long)((g0.y + pa) * p.Wo + (g0.z + pb)) * N;
            long long aoff = -1;
            if (p.add.data) epilogue_row_info(p, row_info(p.rm, r), r, pa, pb, ridx, aoff);
            float* out = p.out + ((size_t)r * (size_t)(p.owy * p.owx) + (size_t)(pa * p.owx + pb)) * N;
#pragma unroll
            for (int n = 0; n < N; ++n) {
                double v = acc[i][n];
                if (aoff >= 0) v += (double)p.add.data[aoff + n];
                if (p.out_grl) v *= (double)relax_factor(v, p.out_grl[ridx + n]);
                out[n] = (float)v;
            }
        }
    }
}

// false: a row's block does not fit the work-group's LDS (the caller takes another form)
static bool launch_cross_image(const CrossParams& p0, hipStream_t s) {
    CrossParams p = p0;
    p.cls_ny = (p.owy + p.sh - 1) / p.sh;
    p.cls_nx = (p.owx + p.sw - 1) / p.sw;
    p.div_cls = make_fastdiv((uint32_t)(p.cls_ny * p.cls_nx));
    p.div_cls_nx = make_fastdiv((uint32_t)p.cls_nx);
    p.div_ntiles_n = make_fastdiv((uint32_t)p.in.C);
    const int ppc = p.cls_ny * p.cls_nx, ncls = p.sh * p.sw;
    const int npix_in = p.in.wy * p.in.wx;
    const int pstride = ((p.in.C + 1) & ~1) + 2;                     // even (16-byte reads), + 2 against bank conflicts
    const long long lds_max = 60 * 1024 / 8;                         // doubles
    const long long r_lds = (lds_max / pstride - 1) / npix_in;
    if (r_lds < 1) return false;
    // rows per work-group: enough items for the four waves (one (class, 64*NIT items) unit each)
    const int per_wave = 64 * IMG_NIT;
    long long R = (long long)per_wave * (ncls >= 4 ? 1 : 4 / ncls) / ppc;
    R = std::max(1ll, std::min(std::min(R, r_lds), (long long)IMG_RMAX));
    const int ngroups = (int)((R * ppc + per_wave - 1) / per_wave);
    const size_t lds = (size_t)(R * npix_in + 1) * pstride * sizeof(double);
    const dim3 grid((unsigned)((p.nrows + R - 1) / R));
    const bool vec = (p.in.C & 3) == 0;
    auto go = [&](auto nn) {
        constexpr int NN = decltype(nn)::value;
        if (vec) hipLaunchKernelGGL((cross_image_kernel<NN, true>), grid, dim3(256), lds, s, p, (int)R, pstride, ngroups);
        else hipLaunchKernelGGL((cross_image_kernel<NN, false>), grid, dim3(256), lds, s, p, (int)R, pstride, ngroups);
    };
    switch (p.Co) {
        case 1: go(std::integral_constant<int, 1>{}); break;
        case 2: go(std::integral_constant<int, 2>{}); break;
        case 3: go(std::integral_constant<int, 3>{}); break;
        default: go(std::integral_constant<int, 4>{}); break;
    }
    return true;
}

// Image layers behind a stride-1 layer with a long K per pixel (3x3 or 5x5 filters over 32 or 64 channels).  With 4 output
// columns a block value feeds only 4 multiply-adds per use, and in the kernels above every output pixel re-loads the
// values under its taps: those steps run at the speed of the vector L1 (64 B/clk), not of the matrix pipe.  Here one
// wave computes a STRIP of P horizontally adjacent output pixels for its 32 rows: a block value (one 16-byte load per
// lane and 16-channel step, as in cross_direct_kernel) is loaded and converted once and used for every output pixel of
// the strip it reaches (up to kw of them), which cuts the L1 traffic and the conversions by that factor.  The filter
// (float64, 4 columns) sits in LDS; its fragments for the kw taps of a filter row are fetched once per (filter row,
// channel step).  Accumulators: one double per lane, 16-row tile and strip pixel (4x4x4 MFMA).
// Requires what the launcher checks: stride 1, every group of 32 consecutive rows at one position of the start layer
// in one box (so the whole geometry is scalar), whole 16-channel steps.
// grid: (row tile of 128 rows, output row, strip) in the XCD-aware order of cross_kernel.
template <int P, int KW>
__global__ __launch_bounds__(256, 2) void cross_strip_kernel(const CrossParams p) {
    constexpr int TM = 2;
    extern __shared__ __attribute__((aligned(16))) double s_w[];          // [tap][4][Ck + 2]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lk = lane >> 4, lm = lane & 15;
    const int Ck = p.in.C, N = p.Co, ldw = Ck + 2;
    const int nstrips = (p.owx + P - 1) / P;
    const uint32_t per_tile = (uint32_t)(p.owy * nstrips);
    const uint32_t total = per_tile * (uint32_t)p.ntiles_m;
    const uint32_t per_xcd = (total + 7u) >> 3;
    const uint32_t logical = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    {   // filter -> LDS (all waves, before any of them leaves)
        const int cnt = p.kh * p.kw * 4 * Ck;
        for (int idx = tid; idx < cnt; idx += 256) {
            const int c = idx % Ck, tn = idx / Ck, n = tn & 3, t = tn >> 2;
            s_w[tn * ldw + c] = n < N ? p.wt64[((size_t)t * N + n) * Ck + c] : 0.0;
        }
        __syncthreads();
    }
    const uint32_t rt = fast_div(logical, p.div_opix);                     // div_opix divides by per_tile here
    const int rem = (int)(logical - rt * per_tile);
    const int pa = rem / nstrips, pb0 = (rem - pa * nstrips) * P;
    const int Pv = min(P, p.owx - pb0);
    const int r_wave = (int)rt * 128 + wave * 32;
    if (r_wave >= p.nrows) return;
    const int rows_here = min(32, p.nrows - r_wave);
    const RowInfo u0 = row_info(p.rm, r_wave), u1 = row_info(p.rm, r_wave + rows_here - 1);
    if (!(u0.b == u1.b && u0.ys == u1.ys && u0.xs == u1.xs)) return;       // excluded by the launcher's conditions
    const int opix = p.owy * p.owx;
    const uint32_t row_elems = (uint32_t)(p.in.wy * p.in.wx * Ck);
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.in.data + (size_t)r_wave * row_elems), 0, (int)((uint32_t)rows_here * row_elems * 4u), 0x00020000);
    // geometry of the wave's common position (scalar)
    const int oiy = clampi(p.in.Sy * u0.ys - p.in.Py, 0, p.in.H - p.in.wy), oix = clampi(p.in.Sx * u0.xs - p.in.Px, 0, p.in.W - p.in.wx);
    const int A = clampi(p.oSy * u0.ys - p.oPy, 0, p.Ho - p.owy) + pa, B0 = clampi(p.oSx * u0.xs - p.oPx, 0, p.Wo - p.owx) + pb0;
    const int ty = p.in.tSy * u0.ys - p.in.tPy, tx = p.in.tSx * u0.xs - p.in.tPx;
    const int ylo = max(max(ty, oiy), 0), yhi = min(min(ty + p.in.tWy, oiy + p.in.wy), p.in.H);
    const int xlo = max(max(tx, oix), 0), xhi = min(min(tx + p.in.tWx, oix + p.in.wx), p.in.W);
    uint32_t a_voff[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rl = i * 16 + lm;
        a_voff[i] = rl < rows_here ? ((uint32_t)rl * row_elems + 4u * (uint32_t)lk) * 4u : kOOB;
    }
    const double* const w_lane = s_w + (lm & 3) * ldw + 4 * lk;
    double acc[TM][P];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int q = 0; q < P; ++q) acc[i][q] = 0.0;

    // tap (f, g) of a stride-1 layer reads, for output pixel (A, B), the layer-output pixel (A + ph - f, B + pw - g);
    // so the block value at (y, x) reaches output pixel B = x - pw + g, i.e. strip pixel q = x - pw + g - B0
    // The strip's block pixels of one filter row are x_j = B0 + pw - (KW-1) + j, j = 0 .. P+KW-2, and x_j reaches strip
    // pixel q = j - (KW-1) + g through tap g: with j and g unrolled every accumulator index is a compile-time constant
    // and a step costs a handful of scalar instructions (the scalar unit is shared by the CU's four SIMDs; with MFMAs
    // of 16 cycles a loop that picks accumulators at run time is bound by it).  Strip pixels beyond the window's edge
    // (last strip) are computed from whatever valid block pixels reach them and not stored.
    // Order of the contributions to one output pixel: filter row, then tap of the row, then channel step - the order
    // cross_direct_kernel uses (its taps ascend, i.e. the block pixels DEscend), with the same instruction on the same
    // operands: a row gets the same bits from either kernel, so results do not depend on which of the two a chunk of
    // rows happens to qualify for.
    constexpr int NJ = P + KW - 1;
    const int xj0 = B0 + p.pw - (KW - 1);
    for (int f = 0; f < p.kh; ++f) {
        const int y = A + p.ph - f;
        if (y < ylo || y >= yhi) continue;
        const uint32_t row_off = (uint32_t)((y - oiy) * p.in.wx - oix) * (uint32_t)Ck;    // + x*Ck + d0 (x >= oix whenever it is used)
        const double* const w_row = w_lane + f * KW * 4 * ldw;
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int j = NJ - 1 - jj;
            const int x = xj0 + j;
            if (x < xlo || x >= xhi) continue;                                      // uniform
            for (int d0 = 0; d0 < Ck; d0 += 16) {
                const uint32_t soff = (row_off + (uint32_t)x * (uint32_t)Ck + (uint32_t)d0) * 4u;
                uint4_t raw[TM];
#pragma unroll
                for (int i = 0; i < TM; ++i) raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soff, 0);
                double bf[KW][4];
#pragma unroll
                for (int g = 0; g < KW; ++g) {
                    const int q = j - (KW - 1) + g;
                    if (q < 0 || q >= P) continue;                                  // compile time
                    const double2* src = reinterpret_cast<const double2*>(w_row + g * 4 * ldw + d0);
                    const double2 v0 = src[0], v1 = src[1];
                    bf[g][0] = v0.x; bf[g][1] = v0.y; bf[g][2] = v1.x; bf[g][3] = v1.y;
                }
                double av[TM][4];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    av[i][0] = (double)__uint_as_float(raw[i].x); av[i][1] = (double)__uint_as_float(raw[i].y);
                    av[i][2] = (double)__uint_as_float(raw[i].z); av[i][3] = (double)__uint_as_float(raw[i].w);
                }
                // k outermost: consecutive MFMAs go to up to KW*TM different accumulators, none waits for the one before
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int g = 0; g < KW; ++g) {
                        const int q = j - (KW - 1) + g;
                        if (q < 0 || q >= P) continue;                              // compile time
#pragma unroll
                        for (int i = 0; i < TM; ++i)
                            acc[i][q] = __builtin_amdgcn_mfma_f64_4x4x4f64(av[i][k], bf[g][k], acc[i][q], 0, 0, 0);
                    }
            }
        }
    }

    // ---- epilogue: the lane's value of tile i is row 4*((l%16)/4) + l/16, column l%4
    const int n = lm & 3;
    const bool has_add = p.add.data != nullptr;
    const int add_oy = has_add ? clampi(p.add.Sy * u0.ys - p.add.Py, 0, p.add.H - p.add.wy) : 0;
    const int add_ox = has_add ? clampi(p.add.Sx * u0.xs - p.add.Px, 0, p.add.W - p.add.wx) : 0;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        if (q >= Pv) continue;
        const int B = B0 + q, pix = pa * p.owx + pb0 + q;
        const long long ridx = (long long)u0.b * ((long long)p.Ho * p.Wo * N) + (long long)(A * p.Wo + B) * N;
        const int ay = A - add_oy, ax = B - add_ox;
        const bool add_in = has_add && ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rl = i * 16 + 4 * (lm >> 2) + lk;
            const int r = r_wave + rl;
            if (r >= p.nrows || n >= N) continue;
            double v = acc[i][q];
            if (add_in) v += (double)p.add.data[((size_t)r * p.add.wy * p.add.wx + (size_t)(ay * p.add.wx + ax)) * N + n];
            if (p.out_grl) v *= (double)relax_factor(v, p.out_grl[ridx + n]);
            p.out[((size_t)r * opix + pix) * N + n] = (float)v;
        }
    }
}

// The strip kernel for 3x3 filters, walking the window: in the kernel above every block row is fetched by the three
// output rows it reaches (three work-groups) and measured HBM traffic is 2.2x the block's bytes at 3.4 TB/s, which is
// what bounds those launches.  Here a work-group owns a strip of P output pixels over the WHOLE height of the window
// and walks the block rows from the bottom of the window up; a block value is loaded and converted once and multiplied
// into the three output rows it reaches (filter rows f = 0, 1, 2 -> output rows y - ph + f), whose accumulators are
// live at the same time; an output row is finished, and stored, after the third block row that reaches it.  Walking UP
// makes an output row receive its filter rows in ascending f, then taps, then channel steps: the order of
// cross_direct_kernel and of the kernel above, with the same instruction on the same operands, so a row gets the same
// bits from any of the three.  The walk is unrolled by three block rows so that the accumulator an output row uses
// (row mod 3) is a compile-time index.
// grid: (row tile of 128 rows, strip) in the XCD-aware order of cross_kernel; p.div_opix divides by the strips per tile.
template <int P>
__global__ __launch_bounds__(256, 2) void cross_stripwalk_kernel(const CrossParams p) {
    constexpr int TM = 2, KW = 3, KH = 3;
    extern __shared__ __attribute__((aligned(16))) double s_w[];          // [tap][4][Ck + 2]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lk = lane >> 4, lm = lane & 15;
    const int Ck = p.in.C, N = p.Co, ldw = Ck + 2;
    const int nstrips = (p.owx + P - 1) / P;
    const uint32_t total = (uint32_t)nstrips * (uint32_t)p.ntiles_m;
    const uint32_t per_xcd = (total + 7u) >> 3;
    const uint32_t logical = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    {   // filter -> LDS (all waves, before any of them leaves)
        const int cnt = KH * KW * 4 * Ck;
        for (int idx = tid; idx < cnt; idx += 256) {
            const int c = idx % Ck, tn = idx / Ck, n = tn & 3, t = tn >> 2;
            s_w[tn * ldw + c] = n < N ? p.wt64[((size_t)t * N + n) * Ck + c] : 0.0;
        }
        __syncthreads();
    }
    const uint32_t rt = fast_div(logical, p.div_opix);
    const int pb0 = (int)(logical - rt * (uint32_t)nstrips) * P;
    const int Pv = min(P, p.owx - pb0);
    const int r_wave = (int)rt * 128 + wave * 32;
    if (r_wave >= p.nrows) return;
    const int rows_here = min(32, p.nrows - r_wave);
    const RowInfo u0 = row_info(p.rm, r_wave), u1 = row_info(p.rm, r_wave + rows_here - 1);
    if (!(u0.b == u1.b && u0.ys == u1.ys && u0.xs == u1.xs)) return;       // excluded by the launcher's conditions
    const int opix = p.owy * p.owx;
    const uint32_t row_elems = (uint32_t)(p.in.wy * p.in.wx * Ck);
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.in.data + (size_t)r_wave * row_elems), 0, (int)((uint32_t)rows_here * row_elems * 4u), 0x00020000);
    // geometry of the wave's common position (scalar)
    const int oiy = clampi(p.in.Sy * u0.ys - p.in.Py, 0, p.in.H - p.in.wy), oix = clampi(p.in.Sx * u0.xs - p.in.Px, 0, p.in.W - p.in.wx);
    const int A0 = clampi(p.oSy * u0.ys - p.oPy, 0, p.Ho - p.owy), B0 = clampi(p.oSx * u0.xs - p.oPx, 0, p.Wo - p.owx) + pb0;
    const int ty = p.in.tSy * u0.ys - p.in.tPy, tx = p.in.tSx * u0.xs - p.in.tPx;
    const int ylo = max(max(ty, oiy), 0), yhi = min(min(ty + p.in.tWy, oiy + p.in.wy), p.in.H);
    const int xlo = max(max(tx, oix), 0), xhi = min(min(tx + p.in.tWx, oix + p.in.wx), p.in.W);
    uint32_t a_voff[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rl = i * 16 + lm;
        a_voff[i] = rl < rows_here ? ((uint32_t)rl * row_elems + 4u * (uint32_t)lk) * 4u : kOOB;
    }
    const double* const w_lane = s_w + (lm & 3) * ldw + 4 * lk;
    double acc[3][TM][P];
#pragma unroll
    for (int sl = 0; sl < 3; ++sl)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 0; q < P; ++q) acc[sl][i][q] = 0.0;
    const int n = lm & 3;
    const bool has_add = p.add.data != nullptr;
    const int add_oy = has_add ? clampi(p.add.Sy * u0.ys - p.add.Py, 0, p.add.H - p.add.wy) : 0;
    const int add_ox = has_add ? clampi(p.add.Sx * u0.xs - p.add.Px, 0, p.add.W - p.add.wx) : 0;
    constexpr int NJ = P + KW - 1;
    const int xj0 = B0 + p.pw - (KW - 1);

    // block row t (relative: y = A0 + ph + t) reaches the window's output rows pa = t + f; C = t mod 3 (compile time)
    auto block_row = [&](int t, auto Cc) {
        constexpr int C = decltype(Cc)::value;
        const int y = A0 + p.ph + t;
        if (y >= ylo && y < yhi) {
            const uint32_t row_off = (uint32_t)((y - oiy) * p.in.wx - oix) * (uint32_t)Ck;
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj) {
                const int j = NJ - 1 - jj;
                const int x = xj0 + j;
                if (x < xlo || x >= xhi) continue;                                      // uniform
                for (int d0 = 0; d0 < Ck; d0 += 16) {
                    const uint32_t soff = (row_off + (uint32_t)x * (uint32_t)Ck + (uint32_t)d0) * 4u;
                    uint4_t raw[TM];
#pragma unroll
                    for (int i = 0; i < TM; ++i) raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, (int)a_voff[i], (int)soff, 0);
                    double av[TM][4];
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        av[i][0] = (double)__uint_as_float(raw[i].x); av[i][1] = (double)__uint_as_float(raw[i].y);
                        av[i][2] = (double)__uint_as_float(raw[i].z); av[i][3] = (double)__uint_as_float(raw[i].w);
                    }
#pragma unroll
                    for (int f = 0; f < KH; ++f) {
                        const int pa = t + f;
                        if (pa < 0 || pa >= p.owy) continue;                            // uniform: window's top and bottom
                        const double* const w_row = w_lane + f * KW * 4 * ldw;
                        double bf[KW][4];
#pragma unroll
                        for (int g = 0; g < KW; ++g) {
                            const int q = j - (KW - 1) + g;
                            if (q < 0 || q >= P) continue;                              // compile time
                            const double2* src = reinterpret_cast<const double2*>(w_row + g * 4 * ldw + d0);
                            const double2 v0 = src[0], v1 = src[1];
                            bf[g][0] = v0.x; bf[g][1] = v0.y; bf[g][2] = v1.x; bf[g][3] = v1.y;
                        }
#pragma unroll
                        for (int k = 0; k < 4; ++k)
#pragma unroll
                            for (int g = 0; g < KW; ++g) {
                                const int q = j - (KW - 1) + g;
                                if (q < 0 || q >= P) continue;                          // compile time
#pragma unroll
                                for (int i = 0; i < TM; ++i)
                                    acc[(C + f) % 3][i][q] =
                                        __builtin_amdgcn_mfma_f64_4x4x4f64(av[i][k], bf[g][k], acc[(C + f) % 3][i][q], 0, 0, 0);
                            }
                    }
                }
            }
        }
        // output row pa = t + 2 has now received its three filter rows: store it and free its accumulators
        const int pa = t + 2;
        if (pa >= 0 && pa < p.owy) {
            const int A = A0 + pa;
#pragma unroll
            for (int q = 0; q < P; ++q) {
                if (q < Pv) {
                    const int B = B0 + q, pix = pa * p.owx + pb0 + q;
                    const long long ridx = (long long)u0.b * ((long long)p.Ho * p.Wo * N) + (long long)(A * p.Wo + B) * N;
                    const int ay = A - add_oy, ax = B - add_ox;
                    const bool add_in = has_add && ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx;
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int rl = i * 16 + 4 * (lm >> 2) + lk;
                        const int r = r_wave + rl;
                        if (r >= p.nrows || n >= N) continue;
                        double v = acc[(C + 2) % 3][i][q];
                        if (add_in) v += (double)p.add.data[((size_t)r * p.add.wy * p.add.wx + (size_t)(ay * p.add.wx + ax)) * N + n];
                        if (p.out_grl) v *= (double)relax_factor(v, p.out_grl[ridx + n]);
                        p.out[((size_t)r * opix + pix) * N + n] = (float)v;
                    }
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[(C + 2) % 3][i][q] = 0.0;
            }
        }
    };
    // relative block rows from the bottom of the window (owy - 1) up to -2, in groups whose first member is 2 (mod 3)
    const int t_first = (p.owy - 1) + (2 - (p.owy - 1) % 3 + 3) % 3;       // smallest t >= owy - 1 with t = 2 (mod 3)
    for (int tt = t_first; tt >= -1; tt -= 3) {
        if (tt <= p.owy - 1) block_row(tt, std::integral_constant<int, 2>{});
        if (tt - 1 <= p.owy - 1) block_row(tt - 1, std::integral_constant<int, 1>{});
        if (tt - 2 <= p.owy - 1 && tt - 2 >= -2) block_row(tt - 2, std::integral_constant<int, 0>{});
    }
}

// does the strip kernel apply?  (stride 1, filter rows of 3 taps, whole channel steps, filter fits in LDS, and every group
// of 32 consecutive rows is one position of the start layer in one box)
static bool strip_applies(const CrossParams& p, size_t& lds) {
    lds = (size_t)p.kh * p.kw * 4 * (p.in.C + 2) * sizeof(double);
    const bool fits = (p.kw == 3 && lds <= 24576) || (p.kw == 5 && lds <= 32768);     // filter rows of 3 or 5 taps
    return p.Co <= 4 && p.wt64 && p.sh == 1 && p.sw == 1 && fits && (p.in.C & 15) == 0 &&
           p.rm.rowid == nullptr && (p.rm.Cs & 31) == 0 && (p.rm.row0 & 31) == 0 && (p.rm.Rc & 31) == 0 && p.owx >= 4;
}

static void launch_cross_strip(const CrossParams& p0, size_t lds, hipStream_t s) {
    constexpr int P = 8;
    CrossParams p = p0;
    p.ntiles_m = (p.nrows + 127) / 128;
    const int nstrips = (p.owx + P - 1) / P;
    p.div_opix = make_fastdiv((uint32_t)(p.owy * nstrips));
    const long long total = (long long)p.ntiles_m * p.owy * nstrips;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    if (p.kw == 3 && p.kh == 3) {       // 3x3: the form that walks the window and reads every block row once
        p.div_opix = make_fastdiv((uint32_t)nstrips);
        const long long wtotal = (long long)p.ntiles_m * nstrips;
        hipLaunchKernelGGL((cross_stripwalk_kernel<P>), dim3((unsigned)(((wtotal + 7) / 8) * 8)), dim3(256), lds, s, p);
        return;
    }
    if (p.kw == 3) hipLaunchKernelGGL((cross_strip_kernel<P, 3>), dim3(blocks), dim3(256), lds, s, p);
    else hipLaunchKernelGGL((cross_strip_kernel<P, 5>), dim3(blocks), dim3(256), lds, s, p);
}

template <int BM, int BN>
static void launch_cross_t(const CrossParams& p0, hipStream_t s) {
    CrossParams p = p0;
    p.ntiles_m = (p.nrows + BM - 1) / BM;
    p.ntiles_n = (p.Co + BN - 1) / BN;
    p.div_ntiles_n = make_fastdiv((uint32_t)p.ntiles_n);
    p.div_opix = make_fastdiv((uint32_t)(p.owy * p.owx));
    const long long total = (long long)p.ntiles_m * p.ntiles_n * p.owy * p.owx;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    // the 16-byte forms read the weights' float64 copy through a 32-bit range; a layer without the copy or beyond
    // that size takes the scalar-load forms, which read the float32 weights
    const bool copy_ok = p.wt64 != nullptr && (long long)p.kh * p.kw * p.Co * p.in.C * 8 < (1ll << 31);
    const bool vec = (p.in.C & 3) == 0 && copy_ok;
    if constexpr (BN >= 32 && BM <= 64) {
        const bool dense = p.kh * p.kw == 1 && p.in.wy * p.in.wx == 1 && p.owy * p.owx == 1 && p.sh == 1 && p.sw == 1 &&
                           p.ph == 0 && p.pw == 0;
        if (dense) {
            if (vec) hipLaunchKernelGGL((cross_kernel<BM, BN, true, true>), dim3(blocks), dim3(256), 0, s, p);
            else hipLaunchKernelGGL((cross_kernel<BM, BN, false, true>), dim3(blocks), dim3(256), 0, s, p);
            return;
        }
    }
    if (vec) hipLaunchKernelGGL((cross_kernel<BM, BN, true, false>), dim3(blocks), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((cross_kernel<BM, BN, false, false>), dim3(blocks), dim3(256), 0, s, p);
}

// ------------------------------------------------------------------------------------------------
// Crossing an average-pooling layer: every channel on its own, the filter is the constant 1/(kh*kw).  Per row the same
// transposed convolution as above (Algorithm 1) without the contraction over channels: a gather of at most
// ceil(kh/sh)*ceil(kw/sw) block entries per new coefficient, so the step is bound by memory, not by arithmetic, and runs
// on plain float64 vector adds.  One lane per (row, window pixel, 4 channels); the lanes of a pixel read consecutive
// channels (16 bytes each).  The sum of the gathered entries is exact in float64 up to (taps - 1) roundings, the scaling
// by the rounded reciprocal adds two more: the caller's slack constant for the step covers taps + 8 of them.
// Epilogue (addend, ReLU substitution, one rounding to float32) as in the other forms.
// A lane works on PX horizontally adjacent window pixels: what depends on the row alone (its position, the window
// origins, the exact window) is worked out once for them (that integer arithmetic, not the memory system, bounds a
// lane-per-pixel version).
// grid: x over (row, window line, group of PX pixels) items, 256 >> lg per work-group; y over chunks of 4 << lg channels.
template <bool VEC, typename CT>
__global__ __launch_bounds__(256) void cross_pool_kernel(const CrossParams p, int lg, FastDiv div_nq, FastDiv div_line) {
    constexpr int PX = 4;
    const int C = p.Co;                                     // channels pass through: p.in.C == p.Co
    const uint32_t nq = div_nq.d, per_row = div_line.d;     // pixel groups per window line, per row (= owy * nq)
    const uint32_t item = blockIdx.x * (256u >> lg) + (threadIdx.x >> lg);
    const int c0 = (int)((blockIdx.y << lg) + (threadIdx.x & ((1u << lg) - 1u))) * 4;
    if (item >= (uint32_t)p.nrows * per_row || c0 >= C) return;
    const uint32_t r = fast_div(item, div_line);
    const uint32_t rem = item - r * per_row;
    const int pa = (int)fast_div(rem, div_nq), pb0 = (int)(rem - (uint32_t)pa * nq) * PX;
    const RowInfo ri = row_info(p.rm, (int)r);
    const int A = clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy) + pa;
    const int B0 = clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx) + pb0;
    // the part of the row's stored window that lies in its exact dependence window (see cross_kernel)
    const int oiy = clampi(p.in.Sy * ri.ys - p.in.Py, 0, p.in.H - p.in.wy), oix = clampi(p.in.Sx * ri.xs - p.in.Px, 0, p.in.W - p.in.wx);
    const int ty = p.in.tSy * ri.ys - p.in.tPy, tx = p.in.tSx * ri.xs - p.in.tPx;
    const int ylo = max(ty, oiy), yhi = min(ty + p.in.tWy, oiy + p.in.wy);
    const int xlo = max(tx, oix), xhi = min(tx + p.in.tWx, oix + p.in.wx);
    const CT* const row = reinterpret_cast<const CT*>(p.in.data) + (size_t)r * (size_t)(p.in.wy * p.in.wx * C) + c0;
    const int nv = min(4, C - c0);
    const int npx = min(PX, p.owx - pb0);
    double acc[PX][4];
#pragma unroll
    for (int q = 0; q < PX; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[q][j] = 0.0;
    // tap (f, g) reads the layer-output pixel ((A + ph - f) / sh, (B + pw - g) / sw) when both divisions are exact
    for (int f = 0; f < p.kh; ++f) {
        const int ny = A + p.ph - f;
        if (ny < 0) break;
        const int y = (int)fast_div((uint32_t)ny, p.div_sh);
        if (y * p.sh != ny || y < ylo || y >= yhi) continue;
        const CT* const line = row + (long long)((y - oiy) * p.in.wx - oix) * C;          // + x * C, x >= oix
#pragma unroll
        for (int q = 0; q < PX; ++q) {
            if (q >= npx) break;
            for (int g = 0; g < p.kw; ++g) {
                const int nx = B0 + q + p.pw - g;
                if (nx < 0) break;
                const int x = (int)fast_div((uint32_t)nx, p.div_sw);
                if (x * p.sw != nx || x < xlo || x >= xhi) continue;
                const CT* a = line + (long long)x * C;
                if (VEC && std::is_same<CT, float>::value) {
                    const float4 v = *reinterpret_cast<const float4*>(a);
                    acc[q][0] += (double)v.x; acc[q][1] += (double)v.y; acc[q][2] += (double)v.z; acc[q][3] += (double)v.w;
                } else if (VEC) {
                    const double2 v0 = reinterpret_cast<const double2*>(a)[0], v1 = reinterpret_cast<const double2*>(a)[1];
                    acc[q][0] += v0.x; acc[q][1] += v0.y; acc[q][2] += v1.x; acc[q][3] += v1.y;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (j < nv) acc[q][j] += (double)a[j];
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < PX; ++q) {
        if (q >= npx) break;
        long long ridx, aoff;
        epilogue_row_info(p, ri, (int)r, pa, pb0 + q, ridx, aoff);
        CT* out = reinterpret_cast<CT*>(p.out) + ((size_t)r * (size_t)(p.owy * p.owx) + (size_t)(pa * p.owx + pb0 + q)) * C + c0;
        CT res[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            res[j] = 0.f;
            if (j < nv) {
                double v = acc[q][j] * p.pool_scale;
                if (aoff >= 0) v += (double)reinterpret_cast<const CT*>(p.add.data)[aoff + c0 + j];
                if (p.out_grl) v *= (double)relax_factor(v, p.out_grl[ridx + c0 + j]);
                res[j] = (CT)v;
            }
        }
        if (VEC && std::is_same<CT, float>::value) {
            *reinterpret_cast<float4*>(out) = make_float4((float)res[0], (float)res[1], (float)res[2], (float)res[3]);
        } else if (VEC) {
            reinterpret_cast<double2*>(out)[0] = make_double2((double)res[0], (double)res[1]);
            reinterpret_cast<double2*>(out)[1] = make_double2((double)res[2], (double)res[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < nv) out[j] = res[j];
        }
    }
}

static void launch_cross_pool(const CrossParams& p, hipStream_t s) {
    const int cg = (p.Co + 3) / 4;                          // groups of 4 channels
    int lg = 0;
    while ((1 << lg) < cg && lg < 6) ++lg;
    const int nq = (p.owx + 3) / 4;
    const long long items = (long long)p.nrows * p.owy * nq;               // < 2^31: rows * window pixels is
    const int per_wg = 256 >> lg;
    const dim3 grid((unsigned)((items + per_wg - 1) / per_wg), (unsigned)((cg + (1 << lg) - 1) >> lg));
    const FastDiv div_nq = make_fastdiv((uint32_t)nq), div_line = make_fastdiv((uint32_t)(p.owy * nq));
    const bool vec = (p.Co & 3) == 0;
    if (p.coef64) {
        if (vec) hipLaunchKernelGGL((cross_pool_kernel<true, double>), grid, dim3(256), 0, s, p, lg, div_nq, div_line);
        else hipLaunchKernelGGL((cross_pool_kernel<false, double>), grid, dim3(256), 0, s, p, lg, div_nq, div_line);
    } else {
        if (vec) hipLaunchKernelGGL((cross_pool_kernel<true, float>), grid, dim3(256), 0, s, p, lg, div_nq, div_line);
        else hipLaunchKernelGGL((cross_pool_kernel<false, float>), grid, dim3(256), 0, s, p, lg, div_nq, div_line);
    }
}

// float64 storage: the general LDS-tiled form for every layer (32 columns per tile when the layer has no more)
template <int BM, int BN>
static void launch_cross_f64_t(const CrossParams& p0, hipStream_t s) {
    CrossParams p = p0;
    p.ntiles_m = (p.nrows + BM - 1) / BM;
    p.ntiles_n = (p.Co + BN - 1) / BN;
    p.div_ntiles_n = make_fastdiv((uint32_t)p.ntiles_n);
    p.div_opix = make_fastdiv((uint32_t)(p.owy * p.owx));
    const long long total = (long long)p.ntiles_m * p.ntiles_n * p.owy * p.owx;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    const bool vec = (p.in.C & 3) == 0;
    const bool dense = p.kh * p.kw == 1 && p.in.wy * p.in.wx == 1 && p.owy * p.owx == 1 && p.sh == 1 && p.sw == 1 &&
                       p.ph == 0 && p.pw == 0;
    const bool copy_ok = p.wt64 != nullptr && (long long)p.Co * p.in.C * 8 < (1ll << 31);   // see launch_cross_t
    if (dense && vec && copy_ok) hipLaunchKernelGGL((cross_kernel<BM, BN, true, true, double>), dim3(blocks), dim3(256), 0, s, p);
    else if (vec) hipLaunchKernelGGL((cross_kernel<BM, BN, true, false, double>), dim3(blocks), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((cross_kernel<BM, BN, false, false, double>), dim3(blocks), dim3(256), 0, s, p);
}
static void launch_cross_f64(const CrossParams& p, hipStream_t s) {
    if (p.Co <= 32) launch_cross_f64_t<64, 32>(p, s);
    else launch_cross_f64_t<64, 64>(p, s);
}

void launch_cross(const CrossParams& p, hipStream_t s) {
    if (p.nrows <= 0 || p.Co <= 0) return;
    if (p.pool_scale != 0.0) { launch_cross_pool(p, s); return; }
    if (p.coef64) { launch_cross_f64(p, s); return; }
    const int N = p.Co;
    // tile shapes measured on MI355X: 64x64 beats the larger tiles (their lower occupancy costs more than their
    // higher arithmetic intensity gains); narrow layers take a tall tile so that fewer MFMA columns are padding
    // narrow layers: no LDS staging, fewer MFMA columns of padding (4-column instruction for the image layers)
    // image layers: one lane per output pixel while the pixel's K (taps of its parity class x channels) is short; a
    // lane's loads are 16 bytes out of a 128-byte line, which the L1 no longer absorbs for longer K (measured: 1.6x
    // faster than the MFMA kernel at K = 64, 0.75x at K = 288)
    const int k_pixel = ((p.kh + p.sh - 1) / p.sh) * ((p.kw + p.sw - 1) / p.sw) * p.in.C;
    if (N <= 4 && p.wt64 && k_pixel <= 128 && launch_cross_image(p, s)) return;
    size_t strip_lds = 0;
    if (N <= 4 && strip_applies(p, strip_lds)) { launch_cross_strip(p, strip_lds, s); return; }
    if (N <= 4) { launch_cross_direct<2, 0>(p, s); return; }
    if (N <= 16) { launch_cross_direct<2, 1>(p, s); return; }
    if (N <= 32) { launch_cross_direct<2, 2>(p, s); return; }
    // few rows (one input at a time): smaller tiles so that the launch still covers the chip
    const long long wg64 = (long long)((p.nrows + 63) / 64) * ((N + 63) / 64) * p.owy * p.owx;
    if (wg64 < 256) { launch_cross_t<32, 32>(p, s); return; }
    if (wg64 < 512) { launch_cross_t<64, 32>(p, s); return; }
    launch_cross_t<64, 64>(p, s);
}

}  // namespace gp
