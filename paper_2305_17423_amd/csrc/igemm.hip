// Gathered implicit GEMM, bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
//   out[row, n] = epilogue( sum_k A[row, k] * W[n, k] )
//
// A rows are gathered on the fly: row -> (b, y, x) of an active pixel, k ->
// (tap, channel) of the (optionally normalised + activated) input maps; nothing
// is packed in HBM.  The workgroup tile is BM x BN with a K step of 32; global
// loads for step i+1 are issued before the MFMAs of step i and land in the other
// half of a double-buffered LDS tile.
#include "igemm.h"

namespace fise {

constexpr int BK = 32;            // K elements per step
constexpr int LDT = BK + 8;       // LDS row pitch in bf16 (80 bytes: keeps 16-byte reads conflict-light)

struct RowInfo { int b, y, x, ok; };

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void igemm_kernel(const IgemmArgs a) {
    static_assert(WGM * WGN == 4, "four waves");
    constexpr int WM = BM / WGM, WN = BN / WGN;        // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;          // 32x32 MFMA blocks per wave
    static_assert(TM >= 1 && TN >= 1, "wave tile too small");
    constexpr int AL = (BM * 4 + 255) / 256;           // 16-byte A loads per thread per step
    constexpr int BL = (BN * 4 + 255) / 256;

    __shared__ __attribute__((aligned(16))) bf16_t As[2][BM][LDT];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN][LDT];
    __shared__ RowInfo rinfo[BM];
    extern __shared__ float2 gn_ss[];                  // [span][Cin] (scale, shift) when a.pro != PRO_NONE

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    const int rows = a.B * a.Ma;
    const int m0 = blockIdx.x * BM;
    const int Cin = a.C0 + a.C1;
    const int pad = a.ksize >> 1;

    // ---- row table
    for (int r = tid; r < BM; r += 256) {
        RowInfo ri; ri.b = 0; ri.y = 0; ri.x = 0; ri.ok = 0;
        const int gm = m0 + r;
        if (gm < rows) {
            ri.ok = 1; ri.b = gm / a.Ma;
            if (a.tile_idx) active_pixel(a.tile_idx, gm % a.Ma, a.tile, a.tiles_w, ri.y, ri.x);
            else ri.x = gm % a.Ma;                      // compact rows: token = position in the batch element
        }
        rinfo[r] = ri;
    }
    // ---- GroupNorm scale/shift table for the batch elements this tile touches
    const int b_first = m0 / a.Ma;
    if (a.pro != PRO_NONE) {
        const int b_last = min(a.B - 1, (m0 + BM - 1) / a.Ma);
        const int cpg = Cin / a.G;
        for (int e = tid; e < (b_last - b_first + 1) * Cin; e += 256) {
            const int bb = b_first + e / Cin, c = e % Cin;
            const float rs = a.gn_rstd[bb * a.G + c / cpg], mu = a.gn_mean[bb * a.G + c / cpg];
            const float sc = rs * bf2f(a.gn_gamma[c]);
            gn_ss[e] = make_float2(sc, bf2f(a.gn_beta[c]) - mu * sc);
        }
    }
    __syncthreads();

    // ---- per-thread load slots
    const int seg = tid & 3;                           // which 8-element segment of the 32-wide K step
    int arow[AL]; bool aok[AL]; int ab[AL], ay[AL], ax[AL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        arow[j] = (tid >> 2) + 64 * j;
        const bool in = arow[j] < BM;
        const RowInfo ri = rinfo[in ? arow[j] : 0];
        aok[j] = in && ri.ok; ab[j] = ri.b; ay[j] = ri.y; ax[j] = ri.x;
    }
    // weight row of tile column j (GEGLU: first half of a wave's columns = value rows, second half = gate rows)
    int brow[BL]; bool bok[BL];
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int col = (tid >> 2) + 64 * j;
        int wr; bool ok = col < BN;
        if (a.geglu) {
            const int wv = col / WN, jj = col % WN, half = jj / (WN / 2), cc = jj % (WN / 2);
            const int oc = blockIdx.y * (BN / 2) + wv * (WN / 2) + cc;
            ok = ok && oc < a.N; wr = oc + half * a.N;
        } else {
            wr = blockIdx.y * BN + col; ok = ok && wr < a.N;
        }
        brow[j] = wr; bok[j] = ok;
    }

    const int nsteps_total = a.K / BK;
    int kc_begin = 0, kc_end = nsteps_total;
    if (a.splits > 1) {
        const int per = (nsteps_total + a.splits - 1) / a.splits;
        kc_begin = blockIdx.z * per; kc_end = min(nsteps_total, kc_begin + per);
    }
    // running (tap, channel) position of the K cursor
    int k0 = kc_begin * BK;
    int tap = k0 / Cin, cc = k0 % Cin;

    uint4 ra[AL], rb[BL];
    auto load_step = [&](int kc) {
        // ---- A
        const int ky = tap / a.ksize, kx = tap % a.ksize;
        const bool second = cc >= a.C0;
        const bf16_t* src = second ? a.a1 : a.a0;
        const int Cs = second ? a.C1 : a.C0;
        const int cs = (second ? cc - a.C0 : cc) + seg * 8;
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (aok[j]) {
                if (a.a_compact) {
                    v = *reinterpret_cast<const uint4*>(src + (size_t)(m0 + arow[j]) * Cs + cs);
                } else {
                    int iy, ix; bool in;
                    if (a.ups) {
                        const int uy = ay[j] + ky - pad, ux = ax[j] + kx - pad;
                        in = uy >= 0 && uy < 2 * a.Hin && ux >= 0 && ux < 2 * a.Win;
                        iy = uy >> 1; ix = ux >> 1;
                    } else {
                        iy = ay[j] * a.stride + ky - pad; ix = ax[j] * a.stride + kx - pad;
                        in = iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win;
                    }
                    if (in) {
                        v = *reinterpret_cast<const uint4*>(src + (((size_t)ab[j] * a.Hin + iy) * a.Win + ix) * Cs + cs);
                        if (a.pro != PRO_NONE) {
                            const float2* ss = gn_ss + (ab[j] - b_first) * Cin + cc + seg * 8;
                            unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float2 s0 = ss[2 * e], s1 = ss[2 * e + 1];
                                float u0 = __uint_as_float(w4[e] << 16) * s0.x + s0.y;
                                float u1 = __uint_as_float(w4[e] & 0xffff0000u) * s1.x + s1.y;
                                if (a.pro == PRO_GN_SILU) { u0 = silu_f(u0); u1 = silu_f(u1); }
                                w4[e] = (unsigned)f2bf(u0) | ((unsigned)f2bf(u1) << 16);
                            }
                            v = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                        }
                    }
                }
            }
            ra[j] = v;
        }
        // ---- B
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (bok[j]) v = *reinterpret_cast<const uint4*>(a.w + (size_t)brow[j] * a.K + (size_t)kc * BK + seg * 8);
            rb[j] = v;
        }
        cc += BK;
        if (cc >= Cin) { cc = 0; ++tap; }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < AL; ++j)
            if (arow[j] < BM) *reinterpret_cast<uint4*>(&As[buf][arow[j]][seg * 8]) = ra[j];
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            const int col = (tid >> 2) + 64 * j;
            if (col < BN) *reinterpret_cast<uint4*>(&Bs[buf][col][seg * 8]) = rb[j];
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    if (kc_begin < kc_end) {
        load_step(kc_begin);
        store_step(0);
        __syncthreads();
        for (int kc = kc_begin; kc < kc_end; ++kc) {
            const int buf = (kc - kc_begin) & 1;
            const bool more = kc + 1 < kc_end;
            if (more) load_step(kc + 1);
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8_t fa[TM], fb[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[i] = *reinterpret_cast<const bf16x8_t*>(&As[buf][wm0 + i * 32 + (lane & 31)][ks * 16 + (lane >> 5) * 8]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[j] = *reinterpret_cast<const bf16x8_t*>(&Bs[buf][wn0 + j * 32 + (lane & 31)][ks * 16 + (lane >> 5) * 8]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
            if (more) store_step(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- split-K: park partial sums; the last workgroup of a tile sums them in split order
    if (a.splits > 1) {
        const int tile_id = blockIdx.y * gridDim.x + blockIdx.x;
        float* mine = a.partial + ((size_t)tile_id * a.splits + blockIdx.z) * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    mine[((wave * TM + i) * TN + j) * 1024 + e * 64 + lane] = acc[i][j][e];
        __threadfence();
        __syncthreads();
        __shared__ int s_last;
        if (tid == 0) s_last = atomicAdd(a.counters + tile_id, 1) == a.splits - 1;
        __syncthreads();
        if (!s_last) return;
        __threadfence();
        const float* base = a.partial + (size_t)tile_id * a.splits * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float s = 0.f;
                    for (int z = 0; z < a.splits; ++z)
                        s += __builtin_nontemporal_load(base + (size_t)z * (BM * BN) + ((wave * TM + i) * TN + j) * 1024 + e * 64 + lane);
                    acc[i][j][e] = s;
                }
        if (tid == 0) a.counters[tile_id] = 0;             // ready for the next launch
    }

    // ---- epilogue
    constexpr int TNE = TN;   // geglu pairs block j with j + TN/2
    const int n_out_blocks = a.geglu ? TNE / 2 : TNE;
#pragma unroll
    for (int j = 0; j < TNE; ++j) {
        if (j >= n_out_blocks) break;
        int col;
        if (a.geglu) col = blockIdx.y * (BN / 2) + (wave % WGN) * (WN / 2) + j * 32 + (lane & 31);
        else col = blockIdx.y * BN + wn0 + j * 32 + (lane & 31);
        if (col >= a.N) continue;
        const float bias_v = a.bias ? bf2f(a.bias[col]) : 0.f;
        const float bias_g = (a.geglu && a.bias) ? bf2f(a.bias[col + a.N]) : 0.f;
        const int sect = col / a.sect_n, scol = col % a.sect_n;
        bf16_t* outp = a.out[sect];
        const int omode = a.out_mode[sect];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = wm0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const RowInfo ri = rinfo[r];
                if (!ri.ok) continue;
                float v = acc[i][j][e] + bias_v;
                if (a.geglu) {
                    const float g = acc[i][(j + TNE / 2) % TNE][e] + bias_g;
                    v = v * (0.5f * g * (1.0f + erff(g * 0.70710678118654752f)));
                }
                if (a.temb) v += a.temb[ri.b * a.temb_stride + col];
                const size_t pix = ((size_t)ri.b * a.Ho + ri.y) * a.Wo + ri.x;
                if (a.res) v += bf2f(a.res_compact ? a.res[(size_t)(m0 + r) * a.N + col] : a.res[pix * a.N + col]);
                if (omode == OUT_COMPACT) outp[(size_t)(m0 + r) * a.sect_n + scol] = f2bf(v);
                else if (omode == OUT_MAP) outp[pix * a.sect_n + scol] = f2bf(v);
                else outp[((size_t)ri.b * a.sect_n + scol) * ((size_t)a.Ho * a.Wo) + (size_t)ri.y * a.Wo + ri.x] = f2bf(v);
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN>
static int launch_cfg(const IgemmArgs& a, hipStream_t st) {
    const int rows = a.B * a.Ma;
    const int ncols = a.geglu ? 2 * a.N : a.N;
    dim3 grid(ceil_div(rows, BM), ceil_div(ncols, BN), a.splits);
    size_t shmem = 0;
    if (a.pro != PRO_NONE) {
        const int span = std::min(a.B, (BM - 1) / a.Ma + 2);
        shmem = (size_t)span * (a.C0 + a.C1) * sizeof(float2);
        constexpr size_t kMaxDyn = 112 * 1024;      // 160 KB of LDS per workgroup minus the static tiles
        if (shmem > kMaxDyn) return fail(FISE_ERR_SHAPE, "igemm: GroupNorm table of %zu bytes does not fit in LDS", shmem);
        static bool raised = false;                 // once: allow more than the default 64 KB of dynamic LDS
        if (!raised) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<BM, BN, WGM, WGN>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxDyn) != hipSuccess)
                return fail(FISE_ERR_HIP, "igemm: cannot raise the dynamic LDS limit");
            raised = true;
        }
    }
    hipLaunchKernelGGL((igemm_kernel<BM, BN, WGM, WGN>), grid, dim3(256), shmem, st, a);
    FISE_CHECK_LAUNCH("igemm");
    return FISE_OK;
}

size_t igemm_workspace_bytes(int rows, int N, int K) {
    (void)rows; (void)N; (void)K;
    return 0;
}

int launch_igemm(const IgemmArgs& a, hipStream_t st) {
    const int rows = a.B * a.Ma;
    if (rows <= 0) return FISE_OK;
    const int Cin = a.C0 + a.C1;
    if (a.K != a.ksize * a.ksize * Cin) return fail(FISE_ERR_SHAPE, "igemm: K=%d != %d*%d*%d", a.K, a.ksize, a.ksize, Cin);
    if (a.C0 % BK || a.C1 % BK) return fail(FISE_ERR_ALIGN, "igemm: channel counts %d,%d must be multiples of %d", a.C0, a.C1, BK);
    if (a.a_compact && (a.ksize != 1 || a.C1 != 0)) return fail(FISE_ERR_SHAPE, "igemm: compact A needs ksize 1, one source");
    if (a.pro != PRO_NONE && (a.G < 1 || Cin % a.G)) return fail(FISE_ERR_SHAPE, "igemm: Cin=%d %% G=%d", Cin, a.G);
    if (a.nsect < 1 || a.nsect > 3 || a.nsect * a.sect_n != a.N) return fail(FISE_ERR_SHAPE, "igemm: sections");
    if (a.splits != 1) return fail(FISE_ERR_SHAPE, "igemm: split-K not enabled");
    if (a.geglu) return launch_cfg<64, 128, 2, 2>(a, st);
    return launch_cfg<64, 64, 2, 2>(a, st);
}

}  // namespace fise
