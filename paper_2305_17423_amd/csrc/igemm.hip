// Gathered implicit GEMM, bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
//   out[row, n] = epilogue( sum_k A[row, k] * W[n, k]  (+ sum_k A2[row, k] * W2[n, k]) )
//
// A rows are gathered on the fly: row -> (b, y, x) of an active pixel, k ->
// (tap, channel) of the (optionally normalised + activated) input maps; nothing
// is packed in HBM.  The optional second product is a 1x1 convolution of other
// maps at the same pixel (the ResNet shortcut), accumulated into the same tile.
//
// The masked problems are small (a few GFLOP, often a few dozen rows against tens
// of MB of weights), so both kernels here are built to keep memory requests in
// flight rather than to maximise MFMA issue: the K loop moves 64 elements per step,
// loads run ahead of the MFMAs (igemm_dma_kernel: straight into an LDS ring;
// igemm_kernel: through a register FIFO, which lets it apply a GroupNorm prologue),
// several workgroups share a CU, and long K loops are split over workgroups
// (partials parked in a workspace and summed in split order by a second launch, so
// the result is deterministic).
#include <algorithm>
#include <cstdlib>
#include "igemm.h"
#include "profile.h"

namespace fise {

constexpr int PF = 2;                   // prefetch distance in K steps (register-staged kernel)
constexpr int NST_RING = 3;             // LDS ring stages of the LDS-direct kernel (2 and 4 measured slower)

struct RowInfo { int b, y, x, ok; };

// Barrier for LDS hand-over only: waits for this wave's LDS traffic, not for its global loads in
// flight (a full __syncthreads() would drain the prefetch FIFO at every step).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Waits until at most N of this wave's vector memory loads are outstanding, then joins the workgroup barrier.
template <int N>
__device__ __forceinline__ void wait_loads() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// A pointer that went through an integer or an opaque register copy has lost the fact that it points to global
// memory; accesses through it would become FLAT instructions (aperture check, both wait counters).  Every access of
// the epilogues says so again.
template <typename T>
__device__ __forceinline__ __attribute__((address_space(1))) T* as_global(T* p) {   // a pointer rebuilt from integers has
    return (__attribute__((address_space(1))) T*)p;                                  // to be told it is global again
}
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));       // plain vectors: the HIP vector classes cannot be
typedef float f32x4v_t __attribute__((ext_vector_type(4)));         // assigned through an address-space pointer
// Epilogue terms that depend on the output position: time projection and residual for output element
// (row gm = (b, y, x), column col).
__device__ __forceinline__ float epilogue_terms(const IgemmArgs& a, int gm, int b, int y, int x, int col) {
    float v = 0.f;
    if (a.temb) v += as_global(a.temb)[b * a.temb_stride + col];
    if (a.res) {
        if (a.res_compact == 2) v += as_global(reinterpret_cast<const float*>(a.res))[(size_t)gm * a.N + col];
        else if (a.res_compact) v += bf2f(as_global(a.res)[(size_t)gm * a.N + col]);
        else v += bf2f(as_global(a.res)[(((size_t)b * a.Ho + y) * a.Wo + x) * a.N + col]);
    }
    return v;
}

// Position of an output row on its map, worked out once per row: pix = (b * Ho + y) * Wo + x, yx = y * Wo + x.
// 24-bit multiplies are exact here (coordinates and map edges are far below 2^24) and run at full rate.
struct OutPos { int b; unsigned pix, yx; };
__device__ __forceinline__ OutPos out_pos(const IgemmArgs& a, int b, int y, int x) {
    OutPos p;
    p.b = b;
    p.yx = __umul24((unsigned)y, (unsigned)a.Wo) + (unsigned)x;
    p.pix = (unsigned)b * (unsigned)(a.Ho * a.Wo) + p.yx;
    return p;
}

// Time projection and residual for columns col .. col + 3 of output row gm (col % 4 == 0, N % 4 == 0).
__device__ __forceinline__ void epilogue_terms4(const IgemmArgs& a, int gm, const OutPos& p, int col, float (&t)[4]) {
    t[0] = t[1] = t[2] = t[3] = 0.f;
    if (a.temb) {
        auto e = as_global(a.temb + (size_t)p.b * a.temb_stride + col);
        t[0] = e[0]; t[1] = e[1]; t[2] = e[2]; t[3] = e[3];
    }
    if (a.res) {
        if (a.res_compact == 2) {
            const f32x4v_t r = *as_global(reinterpret_cast<const f32x4v_t*>(reinterpret_cast<const float*>(a.res) + (size_t)gm * a.N + col));
            t[0] += r[0]; t[1] += r[1]; t[2] += r[2]; t[3] += r[3];
        } else {
            const size_t row = a.res_compact ? (size_t)gm : (size_t)p.pix;
            const u32x2_t r = *as_global(reinterpret_cast<const u32x2_t*>(a.res + row * a.N + col));
            t[0] += __uint_as_float(r[0] << 16); t[1] += __uint_as_float(r[0] & 0xffff0000u);
            t[2] += __uint_as_float(r[1] << 16); t[3] += __uint_as_float(r[1] & 0xffff0000u);
        }
    }
}

// The destinations of the (up to three) column sections.  Indexing a.out[] / a.out_mode[] with a per-lane section
// number makes the compiler build a table: either it selects the ADDRESS inside the kernel-argument block and fetches
// pointer and mode with a vector load (an exposed round trip in front of every store), or it parks the table in LDS,
// which drags in a read of the dispatch packet in host memory for the workgroup size.  So the choice is made with
// arithmetic on the values: base + (col >= n ? d1 : 0) + (col >= 2n ? d2 : 0).
struct OutSel { unsigned long long base, d1, d2; int mode0, m1, m2; int sect_n; };
__device__ __forceinline__ OutSel out_sel(const IgemmArgs& a) {
    OutSel o;
    const unsigned long long p0 = reinterpret_cast<unsigned long long>(a.out[0]), p1 = reinterpret_cast<unsigned long long>(a.out[1]),
                             p2 = reinterpret_cast<unsigned long long>(a.out[2]);
    o.base = p0; o.d1 = p1 - p0; o.d2 = p2 - p1;
    o.mode0 = a.out_mode[0]; o.m1 = a.out_mode[1] - a.out_mode[0]; o.m2 = a.out_mode[2] - a.out_mode[1];
    o.sect_n = a.sect_n;
    return o;
}

// Four consecutive columns col .. col + 3 of one section (col % 4 == 0, section widths are multiples of 4).
// vss: the view tables of this item when the caller has fetched them ahead (null: fetched here)
__device__ __forceinline__ void epilogue_put4(const IgemmArgs& a, const OutSel& o, int gm, const OutPos& p, int col, const float (&v)[4],
                                              const ViewSS* vss = nullptr) {
    // at most three sections: two compares instead of a division
    const bool s1 = col >= o.sect_n, s2 = col >= 2 * o.sect_n;
    const int scol = col - ((int)s1 + (int)s2) * o.sect_n;
    bf16_t* const outp = reinterpret_cast<bf16_t*>(o.base + (s1 ? o.d1 : 0ull) + (s2 ? o.d2 : 0ull));
    const int omode = o.mode0 + (s1 ? o.m1 : 0) + (s2 ? o.m2 : 0);
    if (omode == OUT_TOKENS_T) {
        const size_t HW = (size_t)a.Ho * a.Wo;
        auto q0 = as_global(outp + ((size_t)p.b * o.sect_n + scol) * HW + p.yx);
#pragma unroll
        for (int q = 0; q < 4; ++q) q0[q * HW] = f2bf(v[q]);
        return;
    }
    const u32x2_t packed = {f2bf2(v[0], v[1]), f2bf2(v[2], v[3])};
    if (omode == OUT_COMPACT_F32) {
        const f32x4v_t full = {v[0], v[1], v[2], v[3]};
        *as_global(reinterpret_cast<f32x4v_t*>(reinterpret_cast<float*>(outp) + (size_t)gm * o.sect_n + scol)) = full;
        if (a.mirror) *as_global(reinterpret_cast<u32x2_t*>(a.mirror + (size_t)gm * o.sect_n + scol)) = packed;
    } else if (omode == OUT_COMPACT) {
        *as_global(reinterpret_cast<u32x2_t*>(outp + (size_t)gm * o.sect_n + scol)) = packed;
    } else {
        *as_global(reinterpret_cast<u32x2_t*>(outp + (size_t)p.pix * o.sect_n + scol)) = packed;
        if (a.nview) {
            if (vss) put_views4(a.view, a.nview, p.pix, scol, v, *vss);
            else put_views4(a.view, a.nview, p.b, p.pix, scol, v);
        }
    }
}

// Row table of a tile: output row m0 + r -> (batch element, y, x) of its active pixel (or compact token).
template <int BM, int NT>
__device__ __forceinline__ void build_row_table(const IgemmArgs& a, int m0, int rows, RowInfo* rinfo, int tid) {
    for (int r = tid; r < BM; r += NT) {
        RowInfo ri; ri.b = 0; ri.y = 0; ri.x = 0; ri.ok = 0;
        const int gm = m0 + r;
        if (gm < rows) {
            ri.ok = 1; ri.b = gm / a.Ma;
            if (a.tile_idx && (a.need_pix || !a.a_compact)) active_pixel(a.tile_idx, gm % a.Ma, a.tile, a.tile_w, a.tiles_w, ri.y, ri.x);
            else ri.x = gm % a.Ma;                      // compact rows: token = position in the batch element
        }
        rinfo[r] = ri;
    }
}

// Weight row behind tile column `col` of column tile `by` (-1: past the last output column).
// GEGLU: the first half of a wave's columns are value rows, the second half the matching gate rows.
template <int BN, int WN>
__device__ __forceinline__ int weight_row(const IgemmArgs& a, int by, int col) {
    if (col >= BN) return -1;
    if (a.geglu) {
        const int wv = col / WN, jj = col % WN, half = jj / (WN / 2), cc = jj % (WN / 2);
        const int oc = by * (BN / 2) + wv * (WN / 2) + cc;
        return oc < a.N ? oc + half * a.N : -1;
    }
    const int wr = by * BN + col;
    return wr < a.N ? wr : -1;
}

// What a workgroup does with its accumulators.  Split-K: park them as partial[bz][row][weight row]; a
// second small kernel adds them up in split order and applies the epilogue.  (Handing the partials
// over inside the GEMM kernel needs either device-scope fences, which write back and invalidate
// whole L2s, or L2-bypassing accesses, which measured slower than the extra launch.)  Otherwise:
// bias, GEGLU gate, time projection, residual, store.
template <int BM, int BN, int WGM, int WGN>
__device__ __forceinline__ void finish_tile(const IgemmArgs& a, f32x16_t (&acc)[BM / WGM / 32][BN / WGN / 32], const RowInfo* rinfo,
                                            int m0, int by, int bz, int rows, int lane, int wave, float* stage = nullptr) {
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    if (a.splits > 1) {
        const int ncols = a.geglu ? 2 * a.N : a.N;
        auto P = as_global(a.partial + (size_t)bz * rows * ncols);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int wr = weight_row<BN, WN>(a, by, wn0 + j * 32 + (lane & 31));
            if (wr < 0) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int r = wm0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                    if (m0 + r < rows) P[(size_t)(m0 + r) * ncols + wr] = acc[i][j][e];
                }
        }
        return;
    }
    constexpr int n_out_blocks = TN >= 2 ? TN / 2 : 1;    // GEGLU pairs block j (value) with block j + TN/2 (gate)
    if (stage && (a.N & 3) == 0 && (a.sect_n & 3) == 0) {
        // The finished tile goes through LDS (`stage`: free once every wave has left the K loop) so that the stores
        // are row-contiguous: a thread then owns four consecutive columns of one row, works out that row's
        // destination once and moves 8 or 16 bytes per access, where the accumulator layout would give it one
        // element of sixteen different rows.
        constexpr int NT = 64 * WGM * WGN;
        const int tid = wave * 64 + lane;
        const int OW = a.geglu ? BN / 2 : BN;             // output columns of the tile
        constexpr int pitch = BN + 4;                      // floats per staged row (GEGLU tiles use the first half)
        __syncthreads();                                   // all waves are done reading the operand ring
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (a.geglu && j >= n_out_blocks) break;
            int col, c;                                    // global column, column within the tile
            if (a.geglu) { c = (wave % WGN) * (WN / 2) + j * 32 + (lane & 31); col = by * (BN / 2) + c; }
            else { c = wn0 + j * 32 + (lane & 31); col = by * BN + c; }
            float bias_v = 0.f, bias_g = 0.f;
            if (col < a.N) {
                if (a.bias) bias_v = bf2f(as_global(a.bias)[col]);
                if (a.bias2) bias_v += bf2f(as_global(a.bias2)[col]);
                if (a.geglu && a.bias) bias_g = bf2f(as_global(a.bias)[col + a.N]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int r = wm0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                    float v = acc[i][j][e] + bias_v;
                    if (a.geglu) {
                        const float g = acc[i][(j + TN / 2) % TN][e] + bias_g;
                        v = v * (0.5f * g * (1.0f + erff(g * 0.70710678118654752f)));
                    }
                    stage[r * pitch + c] = v;
                }
        }
        __syncthreads();
        const int cshift = a.geglu ? __builtin_ctz(BN / 8) : __builtin_ctz(BN / 4);   // log2 of the four-column chunks per row
        constexpr int MAXI = (BM * BN / 4 + NT - 1) / NT;
        // Every LDS read of the pass is issued before anything branches on its result (rows and columns past the
        // tile are clamped for the read and masked at the store): the round trips overlap instead of queueing
        // behind one another.  Then every global load (the output may alias the residual), then every store.
        const OutSel osel = out_sel(a);
        RowInfo ri[MAXI]; float4 sv[MAXI]; int colv[MAXI], rowv[MAXI];
#pragma unroll
        for (int it = 0; it < MAXI; ++it) {
            const int item = tid + it * NT;
            const int r = item >> cshift, c = (item - (r << cshift)) * 4;
            rowv[it] = r; colv[it] = by * OW + c;
            const int rc = min(r, BM - 1);
            ri[it] = rinfo[rc];
            sv[it] = *reinterpret_cast<const float4*>(&stage[rc * pitch + c]);
        }
        OutPos pos[MAXI]; bool ok[MAXI];
#pragma unroll
        for (int it = 0; it < MAXI; ++it) {
            ok[it] = rowv[it] < BM && colv[it] < a.N && ri[it].ok;
            pos[it] = out_pos(a, ri[it].b, ri[it].y, ri[it].x);
        }
        if (!a.temb && osel.sect_n >= a.N && osel.mode0 != OUT_TOKENS_T) {
            // The common cases: one destination (bf16 map / bf16 rows / float rows with a bf16 mirror), optional residual
            // (bf16 map or rows, float rows), no time projection.  Everything uniform is decided out here; an item is
            // then one multiply-add for its address, one residual load, the packs and one or two stores.
            const bool out_map = osel.mode0 == OUT_MAP, out_f32 = osel.mode0 == OUT_COMPACT_F32;
            const int resk = !a.res ? 0 : (a.res_compact == 2 ? 2 : 1);
            const bool res_map = a.res_compact == 0;
            u32x2_t rh[MAXI]; f32x4v_t rf[MAXI];
#pragma unroll
            for (int it = 0; it < MAXI; ++it) { rh[it] = u32x2_t{0u, 0u}; rf[it] = f32x4v_t{0.f, 0.f, 0.f, 0.f}; }
            // residual loads without a branch each (a masked-off item reads element 0 instead: valid memory, value
            // unused), so that they all go out back to back
            if (resk == 1) {
                auto src = as_global(reinterpret_cast<const u32x2_t*>(a.res));
#pragma unroll
                for (int it = 0; it < MAXI; ++it) {
                    const size_t e4 = ((res_map ? (size_t)pos[it].pix : (size_t)(m0 + rowv[it])) * a.N + colv[it]) >> 2;
                    rh[it] = src[ok[it] ? e4 : 0];
                }
            } else if (resk == 2) {
                auto src = as_global(reinterpret_cast<const f32x4v_t*>(a.res));
#pragma unroll
                for (int it = 0; it < MAXI; ++it) {
                    const size_t e4 = ((size_t)(m0 + rowv[it]) * a.N + colv[it]) >> 2;
                    rf[it] = src[ok[it] ? e4 : 0];
                }
            }
            // the consumers' scale / shift entries of every item, requested with the residuals (tiles of four items per
            // thread on four waves: the others have no registers to spare and fetch them item by item)
            constexpr bool kViewsAhead = NT <= 256 && MAXI <= 4;
            ViewSS vss[kViewsAhead ? MAXI : 1];
            if (kViewsAhead && out_map && a.nview) {
#pragma unroll
                for (int it = 0; it < MAXI; ++it) view_ss_load(a.view, a.nview, ok[it] ? pos[it].b : 0, ok[it] ? colv[it] : 0, vss[it]);
            }
            auto dst16 = as_global(reinterpret_cast<u32x2_t*>(out_f32 ? reinterpret_cast<unsigned long long>(a.mirror) : osel.base));
            auto dst32 = as_global(reinterpret_cast<f32x4v_t*>(osel.base));
            const bool put16 = !out_f32 || a.mirror != nullptr;
#pragma unroll
            for (int it = 0; it < MAXI; ++it) {
                if (!ok[it]) continue;
                // the residual is added as one term, as everywhere else: value + (0 + residual)
                const float v0 = sv[it].x + (rf[it][0] + __uint_as_float(rh[it][0] << 16));
                const float v1 = sv[it].y + (rf[it][1] + __uint_as_float(rh[it][0] & 0xffff0000u));
                const float v2 = sv[it].z + (rf[it][2] + __uint_as_float(rh[it][1] << 16));
                const float v3 = sv[it].w + (rf[it][3] + __uint_as_float(rh[it][1] & 0xffff0000u));
                const size_t e4 = ((out_map ? (size_t)pos[it].pix : (size_t)(m0 + rowv[it])) * a.N + colv[it]) >> 2;
                if (out_f32) dst32[e4] = f32x4v_t{v0, v1, v2, v3};
                if (put16) dst16[e4] = u32x2_t{f2bf2(v0, v1), f2bf2(v2, v3)};
                if (out_map && a.nview) {
                    const float vv[4] = {v0, v1, v2, v3};
                    if (kViewsAhead) put_views4(a.view, a.nview, pos[it].pix, colv[it], vv, vss[it]);
                    else put_views4(a.view, a.nview, pos[it].b, pos[it].pix, colv[it], vv);
                }
            }
            return;
        }
        float t[MAXI][4];
#pragma unroll
        for (int it = 0; it < MAXI; ++it) t[it][0] = t[it][1] = t[it][2] = t[it][3] = 0.f;
        if (a.temb || a.res) {
#pragma unroll
            for (int it = 0; it < MAXI; ++it)
                if (ok[it]) epilogue_terms4(a, m0 + rowv[it], pos[it], colv[it], t[it]);
        }
#pragma unroll
        for (int it = 0; it < MAXI; ++it) {
            if (!ok[it]) continue;
            const float v[4] = {sv[it].x + t[it][0], sv[it].y + t[it][1], sv[it].z + t[it][2], sv[it].w + t[it][3]};
            epilogue_put4(a, osel, m0 + rowv[it], pos[it], colv[it], v);
        }
        return;
    }
    const size_t HW = (size_t)a.Ho * a.Wo;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        if (a.geglu && j >= n_out_blocks) break;
        int col;
        if (a.geglu) col = by * (BN / 2) + (wave % WGN) * (WN / 2) + j * 32 + (lane & 31);
        else col = by * BN + wn0 + j * 32 + (lane & 31);
        if (col >= a.N) continue;
        // everything that depends on the column alone, once: biases, section, destination, residual / projection bases
        float bias_v = a.bias ? bf2f(as_global(a.bias)[col]) : 0.f;
        if (a.bias2) bias_v += bf2f(as_global(a.bias2)[col]);
        const float bias_g = (a.geglu && a.bias) ? bf2f(as_global(a.bias)[col + a.N]) : 0.f;
        const int sect = col / a.sect_n, scol = col - sect * a.sect_n;
        const OutSel osel = out_sel(a);                   // (never index a.out[] by a run-time value: see out_sel)
        bf16_t* const outp = reinterpret_cast<bf16_t*>(osel.base + (sect >= 1 ? osel.d1 : 0ull) + (sect >= 2 ? osel.d2 : 0ull));
        const int omode = osel.mode0 + (sect >= 1 ? osel.m1 : 0) + (sect >= 2 ? osel.m2 : 0);
        // Two passes per 32-row block: first every load (time projection, residual), then every store.  The
        // output may alias the residual (the residual stream is updated in place), so in a single pass the
        // compiler has to keep each load behind the previous store and the 16 round trips add up.
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float t[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = wm0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const RowInfo ri = rinfo[r];
                t[e] = ri.ok ? epilogue_terms(a, m0 + r, ri.b, ri.y, ri.x, col) : 0.f;
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = wm0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const RowInfo ri = rinfo[r];
                if (!ri.ok) continue;
                float v = acc[i][j][e] + bias_v;
                if (a.geglu) {
                    const float g = acc[i][(j + TN / 2) % TN][e] + bias_g;
                    v = v * (0.5f * g * (1.0f + erff(g * 0.70710678118654752f)));
                }
                v += t[e];
                const size_t gm = (size_t)(m0 + r);
                if (omode == OUT_COMPACT_F32) {
                    as_global(reinterpret_cast<float*>(outp))[gm * a.sect_n + scol] = v;
                    if (a.mirror) as_global(a.mirror)[gm * a.sect_n + scol] = f2bf(v);
                } else if (omode == OUT_COMPACT) {
                    as_global(outp)[gm * a.sect_n + scol] = f2bf(v);
                } else if (omode == OUT_MAP) {
                    const size_t pix = ((size_t)ri.b * a.Ho + ri.y) * a.Wo + ri.x;
                    as_global(outp)[pix * a.sect_n + scol] = f2bf(v);
                    if (a.nview) put_views1(a.view, a.nview, ri.b, pix, scol, v);
                } else {
                    as_global(outp)[((size_t)ri.b * a.sect_n + scol) * HW + (size_t)ri.y * a.Wo + ri.x] = f2bf(v);
                }
            }
        }
    }
}

// BK: K elements per step (64, or 32 for channel counts that are not multiples of 64)
// PRO: compiled with the GroupNorm(+SiLU) prologue (the other instantiation carries none of its code)
template <int BM, int BN, int WGM, int WGN, int BK, bool PRO>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_kernel(const IgemmArgs a) {
    constexpr int NT = 64 * WGM * WGN;                 // threads: one wave per (WM x WN) sub-tile
    constexpr int LDT = BK + 8;                        // LDS row pitch in bf16: 16-byte aligned, not a power of two
    constexpr int TPR = BK / 8;                        // threads per tile row (16 bytes each)
    constexpr int RP = NT / TPR;                       // tile rows covered per pass
    constexpr int WM = BM / WGM, WN = BN / WGN;        // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;          // 32x32 MFMA blocks per wave
    static_assert(TM >= 1 && TN >= 1, "wave tile too small");
    constexpr int AL = (BM + RP - 1) / RP;             // 16-byte A loads per thread per step
    constexpr int BL = (BN + RP - 1) / RP;

    __shared__ __attribute__((aligned(16))) bf16_t As[2][BM][LDT];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN][LDT];
    __shared__ RowInfo rinfo[BM];
    extern __shared__ __attribute__((aligned(16))) float2 gn_ss[];                  // [span][Cin] (scale, shift) when a.pro != PRO_NONE

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    const int rows = a.B * a.Ma;
    // ---- workgroup -> (row tile bx, column tile by, K split bz).  The grid is one-dimensional and the
    // hardware deals consecutive workgroups round-robin to the 8 XCDs, each with an L2 of its own.
    // Workgroup w is therefore given position (w % 8) * (total / 8) + w / 8 of the (bz, by, bx) order
    // with bx fastest: every XCD works on one contiguous run of that order, so a slice of the weight
    // matrix is pulled into one L2 (two at a run boundary) instead of all eight.
    int bx, by, bz;
    {
        const int total = a.gx * a.gy * a.splits, chunk = total >> 3;
        int w = blockIdx.x;
        if (w < (chunk << 3)) w = (w & 7) * chunk + (w >> 3);
        bx = w % a.gx; const int t = w / a.gx; by = t % a.gy; bz = t / a.gy;
    }
    const int m0 = bx * BM;
    const int Cin = a.C0 + a.C1;
    const int pad = a.ksize >> 1;

    build_row_table<BM, NT>(a, m0, rows, rinfo, tid);
    // ---- K range of this workgroup
    const int nsteps1 = a.K / BK;                      // main product
    const int nsteps_total = nsteps1 + a.K2 / BK;      // + the 1x1 side product
    int kc_begin = 0, kc_end = nsteps_total;
    if (a.splits > 1) {
        const int per = (nsteps_total + a.splits - 1) / a.splits;
        kc_begin = bz * per; kc_end = min(nsteps_total, kc_begin + per);
    }
    // ---- GroupNorm (scale, shift) of the channels this K range touches, for the batch elements of
    // this tile, staged in LDS.  A range shorter than Cin is stored rotated: slot = (c - c_lo) mod Cin.
    const int b_first = m0 / a.Ma;
    int c_lo = 0, clen = Cin;
    if (PRO && a.pro != PRO_NONE) {
        const int k_lo = kc_begin * BK, k_hi = min(kc_end, nsteps1) * BK;
        if (k_hi - k_lo < Cin) { c_lo = k_lo % Cin; clen = max(k_hi - k_lo, 0); }
        const int b_last = min(a.B - 1, (m0 + BM - 1) / a.Ma);
        const int cpg = Cin / a.G;
        for (int e = tid * 2; e < (b_last - b_first + 1) * clen; e += 2 * NT) {   // two entries (16 bytes) per thread
            const int bb = b_first + e / clen;
            int c = c_lo + e % clen; if (c >= Cin) c -= Cin;
            // (scale, shift) per (batch element, channel): u = x * scale + shift is GroupNorm with the given
            // statistics.  Worked out here by every workgroup for its own channels: a separate launch that
            // tabulated them once cost more than it saved.
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const float rs = a.gn_rstd[bb * a.G + (c + q) / cpg], mu = a.gn_mean[bb * a.G + (c + q) / cpg];
                const float sc = rs * bf2f(a.gn_gamma[c + q]);
                gn_ss[e + q] = make_float2(sc, bf2f(a.gn_beta[c + q]) - mu * sc);
            }
        }
    }
    __syncthreads();

    // ---- per-thread load slots: TPR threads per tile row, RP rows per pass
    const int seg = tid % TPR;                         // which 8-element segment of the K step
    const int lrow = tid / TPR;
    bool aok[AL]; int ab[AL], ay[AL], ax[AL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const bool in = lrow + RP * j < BM;
        const RowInfo ri = rinfo[in ? lrow + RP * j : 0];
        aok[j] = in && ri.ok; ab[j] = ri.b; ay[j] = ri.y; ax[j] = ri.x;
    }
    int brow[BL]; bool bok[BL];                        // weight row of tile column j
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int wr = weight_row<BN, WN>(a, by, lrow + RP * j);
        brow[j] = wr < 0 ? 0 : wr; bok[j] = wr >= 0;
    }

    // ---- load cursor.  All address arithmetic that does not change from step to step is done here or
    // when the cursor moves to the next tap; a step itself costs one multiply-add per A slot and one
    // pointer bump per B slot (the K loop is otherwise bound by instruction issue, not by memory).
    //   phase 0: main product (taps x channels of a0 | a1), phase 1: 1x1 side product (s0 | s1)
    const bf16_t* p_a0 = a.a0; const bf16_t* p_a1 = a.a1;   // sources of the current phase
    int p_C0 = a.C0, p_Ct = Cin;                            // channels of the first source / of both
    bool side = false;
    int tap = 0, cc = 0;                                    // tap index, channel cursor within the concatenation
    int pix[AL];                                            // input pixel (or compact row) of the current tap, -1 = none
    int opix[AL];                                           // output pixel: the side product reads its sources there
    const bf16_t* bp[BL];                                   // weight pointer of the step about to be issued
#pragma unroll
    for (int j = 0; j < AL; ++j) opix[j] = aok[j] ? (ab[j] * a.Ho + ay[j]) * a.Wo + ax[j] : -1;
    auto set_tap = [&]() {
        const int ky = tap / a.ksize, kx = tap - ky * a.ksize;
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            int p = -1;
            if (aok[j]) {
                if (a.a_compact) p = m0 + lrow + RP * j;
                else if (a.ups) {
                    const int uy = ay[j] + ky - pad, ux = ax[j] + kx - pad;
                    if (uy >= 0 && uy < 2 * a.Hin && ux >= 0 && ux < 2 * a.Win) p = (ab[j] * a.Hin + (uy >> 1)) * a.Win + (ux >> 1);
                } else {
                    const int iy = ay[j] * a.stride + ky - pad, ix = ax[j] * a.stride + kx - pad;
                    if (iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win) p = (ab[j] * a.Hin + iy) * a.Win + ix;
                }
            }
            pix[j] = p;
        }
    };
    auto enter_side = [&](int c_start) {
        side = true; p_a0 = a.s0; p_a1 = a.s1; p_C0 = a.S0; p_Ct = a.K2; cc = c_start;
#pragma unroll
        for (int j = 0; j < AL; ++j) pix[j] = opix[j];
#pragma unroll
        for (int j = 0; j < BL; ++j) bp[j] = a.w2 + (bok[j] ? (size_t)brow[j] * a.K2 + c_start + seg * 8 : 0);
    };
    if (kc_begin < nsteps1) {
        const int k0 = kc_begin * BK;
        tap = k0 / Cin; cc = k0 - tap * Cin;
        set_tap();
#pragma unroll
        for (int j = 0; j < BL; ++j) bp[j] = a.w + (bok[j] ? (size_t)brow[j] * a.K + k0 + seg * 8 : 0);
    } else {
        enter_side((kc_begin - nsteps1) * BK);
    }
    int kc_next = kc_begin;                                 // the step the cursor points at

    // register FIFO: stage s holds the raw data of K step (kc_begin + i) with i % PF == s
    uint4 ra[PF][AL], rb[PF][BL];
    int st_cc[PF]; unsigned st_in[PF];                 // per stage: slot in the GroupNorm table (-1: none), in-image bits

    // Loads of the next K step into FIFO stage s.  Every slot issues exactly one 16-byte load (rows or
    // taps that do not exist, and steps past the end of the range, read a harmless in-bounds address
    // and are zeroed or ignored later), so the number of loads in flight is the same on every path.
    auto issue = [&](int s) {
        const bool live = kc_next < kc_end;
        const bool second = cc >= p_C0;
        const bf16_t* src = second ? p_a1 : p_a0;
        const int Cs = second ? p_Ct - p_C0 : p_C0;
        const int cs = (second ? cc - p_C0 : cc) + seg * 8;
        unsigned inbits = 0;
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            const bool in = live && pix[j] >= 0;
            const unsigned off = in ? (unsigned)pix[j] * (unsigned)Cs + (unsigned)cs : 0u;
            ra[s][j] = *reinterpret_cast<const uint4*>((in ? src : a.a0) + off);
            inbits |= (in ? 1u : 0u) << j;
        }
#pragma unroll
        for (int j = 0; j < BL; ++j) rb[s][j] = *reinterpret_cast<const uint4*>(live ? bp[j] : a.w);
        st_cc[s] = side ? -1 : (cc >= c_lo ? cc - c_lo : cc - c_lo + Cin);     // slot in the staged table
        st_in[s] = inbits;
        if (live) {
            ++kc_next;
#pragma unroll
            for (int j = 0; j < BL; ++j) bp[j] += bok[j] ? BK : 0;
            cc += BK;
            if (!side) {
                if (kc_next == nsteps1) { if (kc_next < kc_end) enter_side(0); }
                else if (cc >= Cin) { cc = 0; ++tap; set_tap(); }
            }
        }
    };
    // registers of stage s -> LDS buffer `buf`, applying the GroupNorm(+SiLU) prologue to in-image elements
    auto stash = [&](int s, int buf) {
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            uint4 v = ra[s][j];
            const bool in = (st_in[s] >> j) & 1u;
            if (!in) v = make_uint4(0, 0, 0, 0);
            if (PRO && a.pro != PRO_NONE && st_cc[s] >= 0 && in) {
                const float2* ss = gn_ss + (ab[j] - b_first) * clen + st_cc[s] + seg * 8;
                unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float2 s0 = ss[2 * e], s1 = ss[2 * e + 1];
                    float u0 = __uint_as_float(w4[e] << 16) * s0.x + s0.y;
                    float u1 = __uint_as_float(w4[e] & 0xffff0000u) * s1.x + s1.y;
                    if (a.pro == PRO_GN_SILU) { u0 = silu_f(u0); u1 = silu_f(u1); }
                    w4[e] = f2bf2(u0, u1);
                }
                v = make_uint4(w4[0], w4[1], w4[2], w4[3]);
            }
            if (lrow + RP * j < BM) *reinterpret_cast<uint4*>(&As[buf][lrow + RP * j][seg * 8]) = v;
        }
#pragma unroll
        for (int j = 0; j < BL; ++j)
            if (lrow + RP * j < BN) *reinterpret_cast<uint4*>(&Bs[buf][lrow + RP * j][seg * 8]) = bok[j] ? rb[s][j] : make_uint4(0, 0, 0, 0);
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fill the FIFO
#pragma unroll
    for (int s = 0; s < PF; ++s) issue(s);

    for (int kc0 = kc_begin; kc0 < kc_end; kc0 += PF) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int kc = kc0 + s;
            if (kc >= kc_end) break;                   // uniform across the workgroup
            const int buf = s & 1;                     // PF is even: the parity of kc - kc_begin
            stash(s, buf);
            issue(s);
            lds_barrier();
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
        }
    }

    finish_tile<BM, BN, WGM, WGN>(a, acc, rinfo, m0, by, bz, rows, lane, wave, nullptr);
}


// ---------------------------------------------------------------------------
// The same contraction with operands moved HBM/L2 -> LDS by the memory pipeline itself
// (buffer loads with the LDS bit): no staging registers, no LDS stores, and all per-load
// address arithmetic in the instruction (scalar base descriptor + per-lane 32-bit offset +
// scalar K offset).  A K step costs a wave (BM + BN) / (8 waves) loads, its share of LDS reads
// and the MFMAs.  Used for every launch without a GroupNorm prologue whose channel counts are
// multiples of 64; the register-staged kernel above covers the rest.
//
// LDS: a ring of NST stages, each (BM + BN) rows of 64 bf16 (128 bytes, no padding).  One load
// instruction of a wave fills 8 consecutive rows: lane l writes 16 bytes at row l / 8, slot l % 8
// (the hardware fixes that order).  Which 16 bytes of the row a lane fetches is free, so slot p
// of row r holds K segment p ^ ((r >> 1) & 7): the MFMA operand reads (32 rows x one segment per
// half wave) then touch every bank equally.
// Rows that do not exist (past the last row, taps outside the image, weight rows past N) carry an
// offset beyond the descriptor's size: the load returns zeros and touches no memory.
// ---------------------------------------------------------------------------
// LINEAR: compact A rows, one source, no side product (the per-token linears): the cursor is a single K offset.
template <int BM, int BN, int WGM, int WGN, int NST, bool LINEAR>
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN >= 8 ? 4 : 1)) void igemm_dma_kernel(const IgemmArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)    // the buffer-descriptor type and builtins exist in the device pass only
    // Kernel arguments arrive through scalar loads that the compiler places where a field is first used:
    // left alone, the set-up below turns into dozens of dependent round trips to the scalar cache.
    // Naming every field the set-up and the K loop need as an operand of an empty asm statement right
    // here makes their loads one batch with one wait.
    asm volatile("" ::"s"(a.a0), "s"(a.a1), "s"(a.C0), "s"(a.C1), "s"(a.a_compact), "s"(a.Hin), "s"(a.Win), "s"(a.ksize), "s"(a.stride),
                 "s"(a.ups), "s"(a.tile_idx), "s"(a.tile), "s"(a.tile_w), "s"(a.tiles_w), "s"(a.Ho), "s"(a.Wo));
    asm volatile("" ::"s"(a.B), "s"(a.Ma), "s"(a.w), "s"(a.N), "s"(a.K), "s"(a.geglu), "s"(a.s0), "s"(a.s1), "s"(a.S0), "s"(a.S1),
                 "s"(a.w2), "s"(a.K2), "s"(a.splits), "s"(a.partial), "s"(a.gx), "s"(a.gy));
    // ... and what the epilogue needs: fetched there, each group of fields was another exposed round trip
    asm volatile("" ::"s"(a.bias), "s"(a.bias2), "s"(a.temb), "s"(a.temb_stride), "s"(a.res), "s"(a.res_compact), "s"(a.sect_n),
                 "s"(a.out[0]), "s"(a.out[1]), "s"(a.out[2]), "s"(a.out_mode[0]), "s"(a.out_mode[1]), "s"(a.out_mode[2]),
                 "s"(a.mirror), "s"(a.need_pix));
    constexpr int NW = WGM * WGN, NT = 64 * NW;
    constexpr int RB = 8 * NW;                          // tile rows filled by one load slot of the workgroup
    static_assert(BM % RB == 0 && BN % RB == 0, "tile rows must split evenly over the waves");
    constexpr int AL = BM / RB, BL = BN / RB;           // load slots per thread and K step
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
    constexpr int STAGE = (BM + BN) * 128;              // bytes
    constexpr unsigned OOB = 0x80000000u;               // beyond any descriptor (sizes are below 2 GiB)
    constexpr int SRD_FLAGS = 0x00020000;               // raw buffer, 32-bit data format

    extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
    __shared__ RowInfo rinfo[BM];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rows = a.B * a.Ma;
    int bx, by, bz;                                     // see igemm_kernel: XCD-aware workgroup order
    {
        const int total = a.gx * a.gy * a.splits, chunk = total >> 3;
        int w = blockIdx.x;
        if (w < (chunk << 3)) w = (w & 7) * chunk + (w >> 3);
        bx = w % a.gx; const int t = w / a.gx; by = t % a.gy; bz = t / a.gy;
    }
    const int m0 = bx * BM;
    const int Cin = a.C0 + a.C1;
    const int pad = a.ksize >> 1;
    build_row_table<BM, NT>(a, m0, rows, rinfo, tid);

    const int nsteps1 = a.K / 64;                       // main product
    const int nsteps_total = nsteps1 + a.K2 / 64;       // + the 1x1 side product
    int kc_begin = 0, kc_end = nsteps_total;
    if (a.splits > 1) {
        const int per = (nsteps_total + a.splits - 1) / a.splits;
        kc_begin = bz * per; kc_end = min(nsteps_total, kc_begin + per);
    }
    __syncthreads();

    // ---- descriptors of the operand arrays
    const unsigned npix_in = a.a_compact ? (unsigned)rows : (unsigned)(a.B * a.Hin * a.Win);
    const unsigned npix_out = (unsigned)(a.B * a.Ho * a.Wo);
    const __amdgpu_buffer_rsrc_t srd_a0 = __builtin_amdgcn_make_buffer_rsrc((void*)a.a0, 0, (int)(npix_in * a.C0 * 2u), SRD_FLAGS);
    const __amdgpu_buffer_rsrc_t srd_a1 = __builtin_amdgcn_make_buffer_rsrc((void*)a.a1, 0, (int)(a.a1 ? npix_in * a.C1 * 2u : 0u), SRD_FLAGS);
    const __amdgpu_buffer_rsrc_t srd_s0 = __builtin_amdgcn_make_buffer_rsrc((void*)a.s0, 0, (int)(a.s0 ? npix_out * a.S0 * 2u : 0u), SRD_FLAGS);
    const __amdgpu_buffer_rsrc_t srd_s1 = __builtin_amdgcn_make_buffer_rsrc((void*)a.s1, 0, (int)(a.s1 ? npix_out * a.S1 * 2u : 0u), SRD_FLAGS);
    const unsigned wrows = (unsigned)(a.geglu ? 2 * a.N : a.N);
    const __amdgpu_buffer_rsrc_t srd_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)(wrows * (unsigned)a.K * 2u), SRD_FLAGS);
    const __amdgpu_buffer_rsrc_t srd_w2 = __builtin_amdgcn_make_buffer_rsrc((void*)a.w2, 0, (int)(a.w2 ? wrows * (unsigned)a.K2 * 2u : 0u), SRD_FLAGS);

    // ---- per-thread load slots: slot j of this wave fills tile rows j * RB + wave * 8 .. + 8
    const int lr = lane >> 3;                           // row within the 8
    int ab[AL], ay[AL], ax[AL]; bool aok[AL]; unsigned aseg[AL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const int r = j * RB + wave * 8 + lr;
        const RowInfo ri = rinfo[r];
        aok[j] = ri.ok; ab[j] = ri.b; ay[j] = ri.y; ax[j] = ri.x;
        aseg[j] = (unsigned)(((lane & 7) ^ ((r >> 1) & 7)) * 16);
    }
    int brow[BL]; unsigned bseg[BL];
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int r = j * RB + wave * 8 + lr;
        brow[j] = weight_row<BN, WN>(a, by, r);
        bseg[j] = (unsigned)(((lane & 7) ^ ((r >> 1) & 7)) * 16);
    }

    // ---- load cursor (wave-uniform apart from the per-lane offsets va / vb)
    //   phase 0: main product, K = taps x (channels of a0 | a1); phase 1: 1x1 side product over s0 | s1
    bool side = false;
    int tap = 0, cc = 0;                                // tap, channel cursor within the concatenation
    int kc_next = kc_begin;
    int pix[AL], opix[AL];                              // input pixel of the current tap / output pixel (-1: none)
    unsigned va[AL], vb[BL];                            // byte offsets of the lanes' rows in the current source / weights
    unsigned soff_a = 0, soff_b = 0;                    // byte offsets of the K step within a row
    __amdgpu_buffer_rsrc_t cur_a = srd_a0, cur_b = srd_w;
#pragma unroll
    for (int j = 0; j < AL; ++j) opix[j] = aok[j] ? (ab[j] * a.Ho + ay[j]) * a.Wo + ax[j] : -1;
    auto set_tap = [&]() {
        const int ky = tap / a.ksize, kx = tap - ky * a.ksize;
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            int p = -1;
            if (aok[j]) {
                if (a.a_compact) p = m0 + j * RB + wave * 8 + lr;
                else if (a.ups) {
                    const int uy = ay[j] + ky - pad, ux = ax[j] + kx - pad;
                    if (uy >= 0 && uy < 2 * a.Hin && ux >= 0 && ux < 2 * a.Win) p = (ab[j] * a.Hin + (uy >> 1)) * a.Win + (ux >> 1);
                } else {
                    const int iy = ay[j] * a.stride + ky - pad, ix = ax[j] * a.stride + kx - pad;
                    if (iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win) p = (ab[j] * a.Hin + iy) * a.Win + ix;
                }
            }
            pix[j] = p;
        }
    };
    // source, row offsets and K offset of the A operand for the cursor position (side, cc)
    auto set_source = [&]() {
        const int c0 = side ? a.S0 : a.C0, ct = side ? a.K2 : Cin;
        const bool second = cc >= c0;
        const unsigned Cs = (unsigned)(second ? ct - c0 : c0);
        cur_a = side ? (second ? srd_s1 : srd_s0) : (second ? srd_a1 : srd_a0);
        soff_a = (unsigned)(second ? cc - c0 : cc) * 2u;
#pragma unroll
        for (int j = 0; j < AL; ++j) va[j] = pix[j] >= 0 ? (unsigned)pix[j] * Cs * 2u + aseg[j] : OOB;
    };
    auto set_weights = [&](int kstep) {                 // kstep: K step within the current phase
        const unsigned Kw = (unsigned)(side ? a.K2 : a.K);
        cur_b = side ? srd_w2 : srd_w;
        soff_b = (unsigned)kstep * 128u;
#pragma unroll
        for (int j = 0; j < BL; ++j) vb[j] = brow[j] >= 0 ? (unsigned)brow[j] * Kw * 2u + bseg[j] : OOB;
    };
    auto enter_side = [&](int kstep) {
        side = true; cc = kstep * 64;
#pragma unroll
        for (int j = 0; j < AL; ++j) pix[j] = opix[j];
        set_source(); set_weights(kstep);
    };
    if constexpr (LINEAR) {
        cur_a = srd_a0; soff_a = (unsigned)kc_begin * 128u;
#pragma unroll
        for (int j = 0; j < AL; ++j) va[j] = aok[j] ? (unsigned)(m0 + j * RB + wave * 8 + lr) * (unsigned)a.C0 * 2u + aseg[j] : OOB;
        set_weights(kc_begin);
    } else if (kc_begin < nsteps1) {
        const int k0 = kc_begin * 64;
        tap = k0 / Cin; cc = k0 - tap * Cin;
        set_tap(); set_source(); set_weights(kc_begin);
    } else {
        enter_side(kc_begin - nsteps1);
    }

    // Loads of the next K step into ring stage st.  Every call issues exactly AL + BL loads per thread
    // (past the end of the K range they are all out of range: zeros, no memory traffic), so the
    // count of loads in flight is known at every point of the loop.
    auto issue = [&](int st) {
        const bool live = kc_next < kc_end;
        unsigned char* base = ring + st * STAGE + wave * 1024;
#pragma unroll
        for (int j = 0; j < AL; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(cur_a, (__attribute__((address_space(3))) void*)(base + j * RB * 128), 16,
                                                     live ? va[j] : OOB, soff_a, 0, 0);
#pragma unroll
        for (int j = 0; j < BL; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(cur_b, (__attribute__((address_space(3))) void*)(base + (BM + j * RB) * 128), 16,
                                                     live ? vb[j] : OOB, soff_b, 0, 0);
        if (live) {
            ++kc_next; soff_a += 128u; soff_b += 128u;
            if constexpr (LINEAR) return;
            cc += 64;
            if (!side) {
                if (kc_next == nsteps1) { if (kc_next < kc_end) enter_side(0); }
                else if (cc >= Cin) { cc = 0; ++tap; set_tap(); set_source(); }
                else if (cc == a.C0) set_source();
            } else if (cc == a.S0 && cc < a.K2) set_source();
        }
    };

    // ---- LDS read offsets of the MFMA operands within a stage (row r, segment ks * 2 + lane / 32, swizzled)
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    unsigned rda[TM][4], rdb[TN][4];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm0 + i * 32 + (lane & 31), t = (lane >> 5) ^ ((r >> 1) & 7);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) rda[i][ks] = (unsigned)(r * 128 + (((ks * 2) ^ t) * 16));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = wn0 + j * 32 + (lane & 31), t = (lane >> 5) ^ ((r >> 1) & 7);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) rdb[j][ks] = (unsigned)((BM + r) * 128 + (((ks * 2) ^ t) * 16));
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s);         // NST - 1 steps in flight

    for (int kc0 = kc_begin; kc0 < kc_end; kc0 += NST) {
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            if (kc0 + s >= kc_end) break;               // uniform across the workgroup
            // the loads of this step are the oldest (NST - 1) * (AL + BL) in flight per thread: wait until only
            // the younger ones remain, then meet the other waves (their rows of the stage have landed too,
            // and everybody is done reading the stage that is refilled next)
            wait_loads<(NST - 2) * (AL + BL)>();
            const unsigned char* stage = ring + s * STAGE;
            // all operand fragments of the step are requested before the first MFMA: the LDS round trips
            // overlap each other and the matrix pipe instead of alternating with it
            bf16x8_t fa[4][TM], fb[4][TN];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[ks][i] = *reinterpret_cast<const bf16x8_t*>(stage + rda[i][ks]);
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[ks][j] = *reinterpret_cast<const bf16x8_t*>(stage + rdb[j][ks]);
            }
            __builtin_amdgcn_sched_barrier(0);          // keep the scheduler from pairing each read with its MFMA again
            issue((s + NST - 1) % NST);                 // next loads and the cursor's scalar work ride on the LDS latency
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
        }
    }
    wait_loads<0>();                                    // the trailing out-of-range loads still target the ring
    finish_tile<BM, BN, WGM, WGN>(a, acc, rinfo, m0, by, bz, rows, lane, wave, reinterpret_cast<float*>(ring));
#endif
}

// ---------------------------------------------------------------------------
// Wave-split form for the per-token products (1x1 convolutions and linears: one source, no taps).
// One workgroup owns a 32 x BN output tile.  Its NW waves split the K range between them, and each wave runs
// the LDS-direct K loop of igemm_dma_kernel on its own share with a ring of its own: a wave waits only for its
// own loads, there is no barrier in the loop.  The NW partial tiles are then summed through LDS in wave order
// (fixed, so the result is deterministic) and the epilogue runs on the sum.  The K split that keeps many memory
// requests in flight for a few-row problem thus ends inside the launch: no parked partials in HBM, no second launch.
// ---------------------------------------------------------------------------
template <int BN, int NW, int NST>
__global__ __launch_bounds__(64 * NW) void igemm_wsk_kernel(const IgemmArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" ::"s"(a.a0), "s"(a.C0), "s"(a.a_compact), "s"(a.Hin), "s"(a.Win), "s"(a.tile_idx), "s"(a.tile), "s"(a.tile_w),
                 "s"(a.tiles_w), "s"(a.Ho), "s"(a.Wo), "s"(a.B), "s"(a.Ma), "s"(a.w), "s"(a.N), "s"(a.K), "s"(a.geglu), "s"(a.gx), "s"(a.gy));
    asm volatile("" ::"s"(a.bias), "s"(a.bias2), "s"(a.temb), "s"(a.temb_stride), "s"(a.res), "s"(a.res_compact), "s"(a.sect_n),
                 "s"(a.out[0]), "s"(a.out[1]), "s"(a.out[2]), "s"(a.out_mode[0]), "s"(a.out_mode[1]), "s"(a.out_mode[2]),
                 "s"(a.mirror), "s"(a.need_pix));
    constexpr int BM = 32, NT = 64 * NW, TN = BN / 32;
    constexpr int AL = BM / 8, BL = BN / 8;             // 16-byte load slots per lane and K step (a load fills 8 tile rows)
    constexpr int STAGE = (BM + BN) * 128;              // bytes
    constexpr int PITCH = BN + 4;                       // floats per row of a parked partial tile
    constexpr unsigned OOB = 0x80000000u;
    constexpr int SRD_FLAGS = 0x00020000;
    static_assert(NW * NST * STAGE >= NW * BM * PITCH * 4, "the partial tiles reuse the operand rings");

    extern __shared__ __attribute__((aligned(16))) unsigned char ring[];      // [NW][NST][STAGE]
    __shared__ RowInfo rinfo[BM];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rows = a.B * a.Ma;
    int bx, by;                                         // XCD-aware order, row tiles fastest: see igemm_kernel
    {
        const int total = a.gx * a.gy, chunk = total >> 3;
        int w = blockIdx.x;
        if (w < (chunk << 3)) w = (w & 7) * chunk + (w >> 3);
        bx = w % a.gx; by = w / a.gx;
    }
    const int m0 = bx * BM;
    // pixel coordinates are needed only to gather rows from a map or to scatter into one; compact rows in, compact
    // rows out (most per-token products) skip the table
    const bool use_table = a.need_pix || !a.a_compact;
    if (use_table) build_row_table<BM, NT>(a, m0, rows, rinfo, tid);
    const int nsteps = a.K / 64;
    const int per = (nsteps + NW - 1) / NW;
    const int kc_begin = wave * per, kc_end = min(nsteps, kc_begin + per);
    if (use_table) __syncthreads();

    const unsigned npix_in = a.a_compact ? (unsigned)rows : (unsigned)(a.B * a.Hin * a.Win);
    const __amdgpu_buffer_rsrc_t srd_a = __builtin_amdgcn_make_buffer_rsrc((void*)a.a0, 0, (int)(npix_in * (unsigned)a.C0 * 2u), SRD_FLAGS);
    const unsigned wrows = (unsigned)(a.geglu ? 2 * a.N : a.N);
    const __amdgpu_buffer_rsrc_t srd_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)(wrows * (unsigned)a.K * 2u), SRD_FLAGS);

    const int lr = lane >> 3;
    unsigned va[AL], vb[BL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const int r = j * 8 + lr;
        unsigned row = (unsigned)(m0 + r);
        if (!a.a_compact) { const RowInfo ri = rinfo[r]; row = (unsigned)((ri.b * a.Hin + ri.y) * a.Win + ri.x); }
        va[j] = m0 + r < rows ? row * (unsigned)a.C0 * 2u + (unsigned)(((lane & 7) ^ ((r >> 1) & 7)) * 16) : OOB;
    }
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int r = j * 8 + lr;
        const int wr = weight_row<BN, BN>(a, by, r);
        vb[j] = wr >= 0 ? (unsigned)wr * (unsigned)a.K * 2u + (unsigned)(((lane & 7) ^ ((r >> 1) & 7)) * 16) : OOB;
    }
    // ---- this thread's share of the epilogue (four consecutive columns of one row per item): everything it has to
    // fetch (biases, time projection, residual) is requested here, before the K loop, and has long arrived when the
    // sums are ready.  (The residual may be the output itself, updated in place: each element is read and written
    // by this thread only.)
    const bool geglu = a.geglu != 0;
    const int OW = geglu ? BN / 2 : BN;                 // output columns of the tile
    const int cshift = geglu ? __builtin_ctz(BN / 8) : __builtin_ctz(BN / 4);   // log2 of the four-column chunks per row
    constexpr int ITEMS = (BM * BN / 4 + NT - 1) / NT;
    int e_r[ITEMS], e_c[ITEMS]; bool e_ok[ITEMS]; OutPos e_pos[ITEMS];
    u32x2_t e_bias[ITEMS], e_bias2[ITEMS], e_gate[ITEMS], e_res16[ITEMS]; f32x4v_t e_res32[ITEMS], e_temb[ITEMS];
    ViewSS e_vss[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int item = tid + it * NT;
        const int r = item >> cshift, c = (item - (r << cshift)) * 4;
        const int gm = m0 + r, col = by * OW + c;
        e_r[it] = r; e_c[it] = c;
        e_ok[it] = r < BM && gm < rows && col < a.N;
        e_bias[it] = e_bias2[it] = e_gate[it] = e_res16[it] = u32x2_t{0u, 0u};
        e_res32[it] = e_temb[it] = f32x4v_t{0.f, 0.f, 0.f, 0.f};
        e_pos[it] = OutPos{0, 0u, 0u};
        if (!e_ok[it]) continue;
        if (use_table) { const RowInfo ri = rinfo[r]; e_pos[it] = out_pos(a, ri.b, ri.y, ri.x); }
        else e_pos[it].b = gm / a.Ma;
        if (a.bias) e_bias[it] = *as_global(reinterpret_cast<const u32x2_t*>(a.bias + col));
        if (a.bias2) e_bias2[it] = *as_global(reinterpret_cast<const u32x2_t*>(a.bias2 + col));
        if (geglu && a.bias) e_gate[it] = *as_global(reinterpret_cast<const u32x2_t*>(a.bias + col + a.N));
        if (a.temb) e_temb[it] = *as_global(reinterpret_cast<const f32x4v_t*>(a.temb + (size_t)e_pos[it].b * a.temb_stride + col));
        if (a.res) {
            if (a.res_compact == 2) e_res32[it] = *as_global(reinterpret_cast<const f32x4v_t*>(reinterpret_cast<const float*>(a.res) + (size_t)gm * a.N + col));
            else e_res16[it] = *as_global(reinterpret_cast<const u32x2_t*>(a.res + (a.res_compact ? (size_t)gm : (size_t)e_pos[it].pix) * a.N + col));
        }
        if (a.nview) view_ss_load(a.view, a.nview, e_pos[it].b, col, e_vss[it]);
    }

    unsigned soff = (unsigned)kc_begin * 128u;
    int kc_next = kc_begin;
    unsigned char* const my_ring = ring + wave * (NST * STAGE);
    auto issue = [&](int st) {
        const bool live = kc_next < kc_end;
        unsigned char* base = my_ring + st * STAGE;
#pragma unroll
        for (int j = 0; j < AL; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(srd_a, (__attribute__((address_space(3))) void*)(base + j * 1024), 16,
                                                     live ? va[j] : OOB, soff, 0, 0);
#pragma unroll
        for (int j = 0; j < BL; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(srd_w, (__attribute__((address_space(3))) void*)(base + (BM + j * 8) * 128), 16,
                                                     live ? vb[j] : OOB, soff, 0, 0);
        if (live) { ++kc_next; soff += 128u; }
    };

    unsigned rda[4], rdb[TN][4];
    {
        const int r = lane & 31, t = (lane >> 5) ^ ((r >> 1) & 7);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) rda[ks] = (unsigned)(r * 128 + (((ks * 2) ^ t) * 16));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int r = j * 32 + (lane & 31), t = (lane >> 5) ^ ((r >> 1) & 7);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) rdb[j][ks] = (unsigned)((BM + r) * 128 + (((ks * 2) ^ t) * 16));
    }
    f32x16_t acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s);
    for (int kc0 = kc_begin; kc0 < kc_end; kc0 += NST) {
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            if (kc0 + s >= kc_end) break;               // uniform across the wave
            // this wave's own loads of the step have landed (a wave reads only what it fetched itself)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * (AL + BL)) : "memory");
            const unsigned char* stage = my_ring + s * STAGE;
            bf16x8_t fa[4], fb[4][TN];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                fa[ks] = *reinterpret_cast<const bf16x8_t*>(stage + rda[ks]);
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[ks][j] = *reinterpret_cast<const bf16x8_t*>(stage + rdb[j][ks]);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue((s + NST - 1) % NST);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks], fb[ks][j], acc[j], 0, 0, 0);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the trailing out-of-range loads still target the ring
    __syncthreads();                                    // every wave has left its ring
    float* const part = reinterpret_cast<float*>(ring);       // [NW][BM][PITCH]
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
            part[(wave * BM + r) * PITCH + j * 32 + (lane & 31)] = acc[j][e];
        }
    __syncthreads();
    // ---- sum of the partial tiles in wave order, then the epilogue on the operands fetched before the K loop
    const OutSel osel = out_sel(a);
    auto lo = [](unsigned w) { return __uint_as_float(w << 16); };
    auto hi = [](unsigned w) { return __uint_as_float(w & 0xffff0000u); };
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        if (!e_ok[it]) continue;
        const int r = e_r[it], c = e_c[it];
        float v[4] = {0.f, 0.f, 0.f, 0.f}, g[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float4 p = *reinterpret_cast<const float4*>(&part[(w * BM + r) * PITCH + c]);
            v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
            if (geglu) {
                const float4 q = *reinterpret_cast<const float4*>(&part[(w * BM + r) * PITCH + c + BN / 2]);
                g[0] += q.x; g[1] += q.y; g[2] += q.z; g[3] += q.w;
            }
        }
        // same order of additions as the other epilogues: sum, biases, (gate), then time projection + residual as one term
        v[0] += lo(e_bias[it][0]) + lo(e_bias2[it][0]); v[1] += hi(e_bias[it][0]) + hi(e_bias2[it][0]);
        v[2] += lo(e_bias[it][1]) + lo(e_bias2[it][1]); v[3] += hi(e_bias[it][1]) + hi(e_bias2[it][1]);
        if (geglu) {
            g[0] += lo(e_gate[it][0]); g[1] += hi(e_gate[it][0]); g[2] += lo(e_gate[it][1]); g[3] += hi(e_gate[it][1]);
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = v[q] * (0.5f * g[q] * (1.0f + erff(g[q] * 0.70710678118654752f)));
        }
        v[0] += e_temb[it][0] + (e_res32[it][0] + lo(e_res16[it][0])); v[1] += e_temb[it][1] + (e_res32[it][1] + hi(e_res16[it][0]));
        v[2] += e_temb[it][2] + (e_res32[it][2] + lo(e_res16[it][1])); v[3] += e_temb[it][3] + (e_res32[it][3] + hi(e_res16[it][1]));
        epilogue_put4(a, osel, m0 + r, e_pos[it], by * OW + c, v, a.nview ? &e_vss[it] : nullptr);
    }
#endif
}

// Second half of a split-K launch: one thread per four output columns sums the parked partials in
// split order (deterministic) and applies the epilogue.  A kernel this small lives on memory round
// trips, so everything is requested up front: the pixel of the row, then biases, time projection and
// residual, then the partials (16 bytes per split, twice that with the GEGLU gate, four splits in flight).
template <bool GEGLU>
__global__ __launch_bounds__(256) void igemm_reduce_kernel(const IgemmArgs a) {
    // one batch of kernel-argument loads instead of a dependent round trip per group of fields (see igemm_dma_kernel)
    asm volatile("" ::"s"(a.B), "s"(a.Ma), "s"(a.N), "s"(a.partial), "s"(a.splits), "s"(a.bias), "s"(a.bias2), "s"(a.temb),
                 "s"(a.temb_stride), "s"(a.tile_idx), "s"(a.need_pix), "s"(a.tile), "s"(a.tile_w), "s"(a.tiles_w), "s"(a.res),
                 "s"(a.res_compact));
    asm volatile("" ::"s"(a.Ho), "s"(a.Wo), "s"(a.out[0]), "s"(a.out[1]), "s"(a.out[2]), "s"(a.out_mode[0]), "s"(a.out_mode[1]),
                 "s"(a.out_mode[2]), "s"(a.sect_n), "s"(a.mirror));
    const int rows = a.B * a.Ma;
    const int gm = blockIdx.y * 4 + (threadIdx.x >> 6);  // 4 rows per workgroup; 64 threads x 4 columns per row and block
    const int col = (blockIdx.x * 64 + (threadIdx.x & 63)) * 4;
    if (gm >= rows || col >= a.N) return;                // N % 4 == 0 (checked by the launcher)
    const int ncols = GEGLU ? 2 * a.N : a.N;
    const size_t stride = (size_t)rows * ncols;
    const float* P = a.partial + (size_t)gm * ncols + col;
    const int b = gm / a.Ma, m = gm - b * a.Ma;
    const OutSel osel = out_sel(a);
    // Every load that does not depend on another is requested before anything is used: biases, the time
    // projection, the tile id of this row and a compact residual go out together with the first partials.
    // (Used where they are loaded, each would be a round trip of its own in front of the sum.)
    uint2 bias_raw = make_uint2(0u, 0u), bias2_raw = bias_raw, gate_raw = bias_raw, res_raw = bias_raw;
    float4 temb_v = make_float4(0.f, 0.f, 0.f, 0.f), res_v = temb_v;
    if (a.bias) bias_raw = *reinterpret_cast<const uint2*>(a.bias + col);
    if (a.bias2) bias2_raw = *reinterpret_cast<const uint2*>(a.bias2 + col);
    if (GEGLU && a.bias) gate_raw = *reinterpret_cast<const uint2*>(a.bias + col + a.N);
    if (a.temb) {
        const float* e = a.temb + (size_t)b * a.temb_stride + col;
        temb_v = make_float4(e[0], e[1], e[2], e[3]);
    }
    const bool pix = a.tile_idx && a.need_pix;
    const int tt = a.tile * a.tile_w;
    int tile_id = 0;
    if (pix) tile_id = a.tile_idx[m / tt];
    if (a.res && a.res_compact == 2) res_v = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.res) + (size_t)gm * a.N + col);
    else if (a.res && a.res_compact) res_raw = *reinterpret_cast<const uint2*>(a.res + (size_t)gm * a.N + col);
    ViewSS vss;
    if (a.nview) view_ss_load(a.view, a.nview, b, col, vss);       // (normalised copies: one map section, so col is its column)
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f), g = v;
#pragma unroll 4
    for (int z = 0; z < a.splits; ++z) {                  // split order: deterministic; four splits in flight
        const float4 p = *reinterpret_cast<const float4*>(P + z * stride);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        if (GEGLU) { const float4 q = *reinterpret_cast<const float4*>(P + z * stride + a.N); g.x += q.x; g.y += q.y; g.z += q.z; g.w += q.w; }
    }
    // position of the row on the map (needs the tile id), then the one load that depends on it
    int y = 0, x = m;
    if (pix) {
        const int p = m % tt;
        y = (tile_id / a.tiles_w) * a.tile + p / a.tile_w;
        x = (tile_id % a.tiles_w) * a.tile_w + p % a.tile_w;
    }
    const OutPos pos = out_pos(a, b, y, x);
    if (a.res && a.res_compact == 0) res_raw = *reinterpret_cast<const uint2*>(a.res + (size_t)pos.pix * a.N + col);
    auto lo = [](unsigned w) { return __uint_as_float(w << 16); };
    auto hi = [](unsigned w) { return __uint_as_float(w & 0xffff0000u); };
    // same order of additions as the unsplit epilogue: sum, biases, (gate), time projection, residual
    float r[4] = {v.x + (lo(bias_raw.x) + lo(bias2_raw.x)), v.y + (hi(bias_raw.x) + hi(bias2_raw.x)),
                  v.z + (lo(bias_raw.y) + lo(bias2_raw.y)), v.w + (hi(bias_raw.y) + hi(bias2_raw.y))};
    if (GEGLU) {
        const float gg[4] = {g.x + lo(gate_raw.x), g.y + hi(gate_raw.x), g.z + lo(gate_raw.y), g.w + hi(gate_raw.y)};
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = r[q] * (0.5f * gg[q] * (1.0f + erff(gg[q] * 0.70710678118654752f)));
    }
    const float post[4] = {temb_v.x + (res_v.x + lo(res_raw.x)), temb_v.y + (res_v.y + hi(res_raw.x)),
                           temb_v.z + (res_v.z + lo(res_raw.y)), temb_v.w + (res_v.w + hi(res_raw.y))};
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] += post[q];
    epilogue_put4(a, osel, gm, pos, col, r, a.nview ? &vss : nullptr);
}

// Split-K reduce fused with the LayerNorm that follows a residual-stream GEMM: LPR lanes share a row of
// N = 20 * LPR columns (320 / 640 / 1280), each lane owns 20 consecutive columns as 5 x float4.  The
// lanes sum the partials in split order on top of bias and residual, store the float row (the new
// residual stream), then normalise it in registers (two passes, fp32) and store the bf16 LayerNorm row.
template <int LPR>
__global__ __launch_bounds__(256) void igemm_reduce_ln_kernel(const IgemmArgs a) {
    asm volatile("" ::"s"(a.B), "s"(a.Ma), "s"(a.partial), "s"(a.splits), "s"(a.bias), "s"(a.res), "s"(a.out[0]), "s"(a.mirror),
                 "s"(a.ln_gamma), "s"(a.ln_beta), "s"(a.ln_eps), "s"(a.ln_out));    // one batch of argument loads
    constexpr int C = 20 * LPR, RPB = 256 / LPR;
    const int rows = a.B * a.Ma;
    const int row = blockIdx.x * RPB + threadIdx.x / LPR;
    const int l = threadIdx.x % LPR;
    if (row >= rows) return;                      // whole LPR-lane groups leave together
    const size_t off = (size_t)row * C + l * 20;
    // LayerNorm scale and shift of this lane's channels: requested here with everything else (read in the store loop
    // they would each wait behind the previous store, which the compiler must assume may alias them)
    uint2 gv[5], bv[5];
    {
        const uint2* g2 = reinterpret_cast<const uint2*>(a.ln_gamma + l * 20);
        const uint2* b2 = reinterpret_cast<const uint2*>(a.ln_beta + l * 20);
#pragma unroll
        for (int j = 0; j < 5; ++j) { gv[j] = g2[j]; bv[j] = b2[j]; }
    }
    float4 v[5];
    {
        // residual and bias: each as one batch of loads behind one uniform test (tested per element they became
        // five load - wait - add rounds)
        uint2 bb[5];
#pragma unroll
        for (int j = 0; j < 5; ++j) { v[j] = make_float4(0.f, 0.f, 0.f, 0.f); bb[j] = make_uint2(0u, 0u); }
        if (a.res) {
            const float4* r4 = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.res) + off);
#pragma unroll
            for (int j = 0; j < 5; ++j) v[j] = r4[j];
        }
        if (a.bias) {
            const uint2* b2 = reinterpret_cast<const uint2*>(a.bias + l * 20);
#pragma unroll
            for (int j = 0; j < 5; ++j) bb[j] = b2[j];
        }
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            v[j].x += __uint_as_float(bb[j].x << 16); v[j].y += __uint_as_float(bb[j].x & 0xffff0000u);
            v[j].z += __uint_as_float(bb[j].y << 16); v[j].w += __uint_as_float(bb[j].y & 0xffff0000u);
        }
    }
    const float4* P = reinterpret_cast<const float4*>(a.partial + off);
    const size_t stride4 = (size_t)rows * C / 4;
#pragma unroll 4
    for (int z = 0; z < a.splits; ++z) {
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const float4 p = P[z * stride4 + j];
            v[j].x += p.x; v[j].y += p.y; v[j].z += p.z; v[j].w += p.w;
        }
    }
    float4* h4 = reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out[0]) + off);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 5; ++j) { h4[j] = v[j]; s += (v[j].x + v[j].y) + (v[j].z + v[j].w); }
    if (a.mirror) {
        uint2* m2 = reinterpret_cast<uint2*>(a.mirror + off);
#pragma unroll
        for (int j = 0; j < 5; ++j) m2[j] = make_uint2(f2bf2(v[j].x, v[j].y), f2bf2(v[j].z, v[j].w));
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const float mu = s / C;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const float a0 = v[j].x - mu, a1 = v[j].y - mu, a2 = v[j].z - mu, a3 = v[j].w - mu;
        q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) q += __shfl_xor(q, o);
    const float rs = rsqrtf(q / C + a.ln_eps);
    uint2* o2 = reinterpret_cast<uint2*>(a.ln_out + off);
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const float y0 = (v[j].x - mu) * rs * __uint_as_float(gv[j].x << 16) + __uint_as_float(bv[j].x << 16);
        const float y1 = (v[j].y - mu) * rs * __uint_as_float(gv[j].x & 0xffff0000u) + __uint_as_float(bv[j].x & 0xffff0000u);
        const float y2 = (v[j].z - mu) * rs * __uint_as_float(gv[j].y << 16) + __uint_as_float(bv[j].y << 16);
        const float y3 = (v[j].w - mu) * rs * __uint_as_float(gv[j].y & 0xffff0000u) + __uint_as_float(bv[j].y & 0xffff0000u);
        o2[j] = make_uint2(f2bf2(y0, y1), f2bf2(y2, y3));
    }
}


// ---------------------------------------------------------------------------
// host side: tile shape and K split per problem
// ---------------------------------------------------------------------------
size_t igemm_workspace_bytes() { return IGEMM_PARTIAL_BYTES; }

int igemm_workspace_init(void* workspace, size_t bytes, IgemmWorkspace* out, hipStream_t st) {
    (void)st;
    out->partial = nullptr; out->partial_bytes = 0;
    if (!workspace || bytes < igemm_workspace_bytes()) return FISE_OK;          // no split-K without it
    out->partial = (float*)workspace;
    out->partial_bytes = IGEMM_PARTIAL_BYTES;
    return FISE_OK;
}

// How many workgroups share the K loop of one output tile.  A CU pulls operands at a few tens of
// GB/s whatever runs on it, so what matters most is that every CU streams part of the operands: aim
// at roughly two workgroups per CU, keep at least two K steps per workgroup, and keep the parked
// partials (written once, read once by the reduce launch) below the operand traffic.  Measured on
// MI355X, this simple rule beat cost models that tried to price the second launch.
template <int BM, int BN, int BK>
static int pick_splits(const IgemmArgs& a, const IgemmWorkspace* ws, int ncols) {
    if (!ws || !ws->partial) return 1;
    const int rows = a.B * a.Ma;
    const int tiles = ceil_div(rows, BM) * ceil_div(ncols, BN);
    const int nsteps = (a.K + a.K2) / BK;
    constexpr int target = 480;                         // measured optimum is flat between 384 and 480 workgroups
    // Below a dozen K steps the LDS-direct kernel finishes a tile faster alone (6 us + 0.33 us per step) than a
    // split launch and its reduce launch do together; the register-staged kernel has a slower step and splits earlier.
    const int min_steps = a.pro != PRO_NONE ? 4 : 12;
    if (tiles * 2 > target || nsteps < min_steps) return 1;
    const size_t out_bytes = (size_t)rows * ncols * sizeof(float);
    int s = (target + tiles - 1) / tiles;
    s = std::min(s, nsteps / 2);
    s = std::min<int>(s, (int)(ws->partial_bytes / out_bytes));
    const double op_bytes = 2.0 * (double)(a.K + a.K2) * ((double)ncols * ceil_div(rows, BM) + (double)rows * ceil_div(ncols, BN));
    while (s > 1 && 2.0 * s * out_bytes > op_bytes) --s;
    return std::max(s, 1);
}

template <int BM, int BN, int WGM, int WGN, int BK>
static int launch_bk(IgemmArgs a, const IgemmWorkspace* ws, int prof_kind, hipStream_t st) {
    const int rows = a.B * a.Ma;
    const int ncols = a.geglu ? 2 * a.N : a.N;
    a.splits = (a.N % 4 == 0 && a.sect_n % 4 == 0) ? pick_splits<BM, BN, BK>(a, ws, ncols) : 1;
    if (a.splits > 1) a.partial = ws->partial;
    a.gx = ceil_div(rows, BM); a.gy = ceil_div(ncols, BN);
    if (a.tile_w <= 0) a.tile_w = a.tile;
    a.need_pix = a.res && a.res_compact == 0;
    for (int sct = 0; sct < a.nsect; ++sct) a.need_pix |= a.out_mode[sct] == OUT_MAP || a.out_mode[sct] == OUT_TOKENS_T;
    dim3 grid((unsigned)(a.gx * a.gy * a.splits));
    size_t shmem = 0;
    if (a.pro != PRO_NONE) {
        const int span = std::min(a.B, (BM - 1) / a.Ma + 2);
        const int Cin = a.C0 + a.C1;
        const int per = ceil_div((a.K + a.K2) / BK, a.splits);
        shmem = (size_t)span * std::min(Cin, per * BK) * sizeof(float2);
        constexpr size_t kMaxDyn = 64 * 1024;
        if (shmem > kMaxDyn) return fail(FISE_ERR_SHAPE, "igemm: GroupNorm table of %zu bytes does not fit in LDS", shmem);
        // once per instantiation (static tiles + table may exceed 64 KB); a function-local static initialises thread-safely
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<BM, BN, WGM, WGN, BK, true>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxDyn);
        if (attr != hipSuccess) return fail(FISE_ERR_HIP, "igemm: cannot raise the dynamic LDS limit");
    }
    const double flops = 2.0 * rows * (double)ncols * ((double)a.K + a.K2);
    const double bytes = 2.0 * ((double)ncols * ((double)a.K + a.K2) + (double)rows * (a.C0 + a.C1 + a.S0 + a.S1) + (double)rows * a.N);
    // LDS-direct kernel: needs 64-wide K steps, no prologue, and every operand array below 2 GiB (32-bit
    // buffer offsets with the top bit reserved for "no such row")
    constexpr size_t kLim = (size_t)1 << 31;
    const size_t npix_in = a.a_compact ? (size_t)rows : (size_t)a.B * a.Hin * a.Win, npix_out = (size_t)a.B * a.Ho * a.Wo;
    const bool dma = BK == 64 && a.pro == PRO_NONE && npix_in * std::max(a.C0, a.C1) * 2 < kLim &&
                     npix_out * std::max(a.S0, a.S1) * 2 < kLim && (size_t)ncols * std::max(a.K, a.K2) * 2 < kLim;
    if (dma) {
        constexpr int NST = NST_RING;
        constexpr int ring = NST * (BM + BN) * 128;
        static const bool raised = ring <= 48 * 1024 ||        // once per instantiation, thread-safe
            (hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_dma_kernel<BM, BN, WGM, WGN, NST, false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, ring) == hipSuccess &&
             hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_dma_kernel<BM, BN, WGM, WGN, NST, true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, ring) == hipSuccess);
        if (!raised) return fail(FISE_ERR_HIP, "igemm: cannot raise the dynamic LDS limit");
        ProfileScope prof(prof_kind, flops, bytes, st);      // brackets the GEMM launch alone
        if (a.a_compact && a.K2 == 0)
            hipLaunchKernelGGL((igemm_dma_kernel<BM, BN, WGM, WGN, NST, true>), grid, dim3(64 * WGM * WGN), ring, st, a);
        else
            hipLaunchKernelGGL((igemm_dma_kernel<BM, BN, WGM, WGN, NST, false>), grid, dim3(64 * WGM * WGN), ring, st, a);
    } else {
        ProfileScope prof(PROF_IGEMM_STAGED, flops, bytes, st);
        if (a.pro != PRO_NONE) hipLaunchKernelGGL((igemm_kernel<BM, BN, WGM, WGN, BK, true>), grid, dim3(64 * WGM * WGN), shmem, st, a);
        else hipLaunchKernelGGL((igemm_kernel<BM, BN, WGM, WGN, BK, false>), grid, dim3(64 * WGM * WGN), 0, st, a);
    }
    FISE_CHECK_LAUNCH("igemm");
    // LayerNorm of the finished rows: inside the reduce launch when there is one and the row shape is one the
    // fused kernel is built for, otherwise as a launch of its own after the rows are complete
    const bool ln = a.ln_out != nullptr;
    if (ln && (a.nsect != 1 || a.out_mode[0] != OUT_COMPACT_F32 || a.geglu || !a.ln_gamma || !a.ln_beta))
        return fail(FISE_ERR_SHAPE, "igemm: LayerNorm output needs one float compact section");
    const bool ln_fused = ln && a.splits > 1 && !a.temb && !a.bias2 && (!a.res || a.res_compact == 2) &&
                          (a.N == 320 || a.N == 640 || a.N == 1280);
    if (ln_fused) {
        ProfileScope prof(PROF_REDUCE, 0.0, (double)a.splits * rows * ncols * 4.0 + 10.0 * rows * a.N, st);
        if (a.N == 320) hipLaunchKernelGGL(igemm_reduce_ln_kernel<16>, dim3(ceil_div(rows, 16)), dim3(256), 0, st, a);
        else if (a.N == 640) hipLaunchKernelGGL(igemm_reduce_ln_kernel<32>, dim3(ceil_div(rows, 8)), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(igemm_reduce_ln_kernel<64>, dim3(ceil_div(rows, 4)), dim3(256), 0, st, a);
        FISE_CHECK_LAUNCH("igemm reduce + layernorm");
        return FISE_OK;
    }
    if (a.splits > 1) {
        const dim3 rgrid((unsigned)ceil_div(a.N / 4, 64), (unsigned)ceil_div(rows, 4));
        ProfileScope prof(PROF_REDUCE, 0.0, (double)a.splits * rows * ncols * 4.0 + 2.0 * rows * a.N, st);
        if (a.geglu) hipLaunchKernelGGL(igemm_reduce_kernel<true>, rgrid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL(igemm_reduce_kernel<false>, rgrid, dim3(256), 0, st, a);
        FISE_CHECK_LAUNCH("igemm reduce");
    }
    if (ln) return launch_ln_rows(a.out[0], 1, rows, a.N, a.ln_gamma, a.ln_beta, a.ln_eps, a.ln_out, nullptr, 1, 1, 1, 1, 1, st);
    return FISE_OK;
}

template <int BM, int BN, int WGM, int WGN>
static int launch_cfg(const IgemmArgs& a, const IgemmWorkspace* ws, int prof_kind, hipStream_t st) {
    const bool k64 = a.C0 % 64 == 0 && a.C1 % 64 == 0 && a.S0 % 64 == 0 && a.S1 % 64 == 0;
    if (k64) return launch_bk<BM, BN, WGM, WGN, 64>(a, ws, prof_kind, st);
    return launch_bk<BM, BN, WGM, WGN, 32>(a, ws, prof_kind, st);
}

// ---- launcher of the wave-split form
constexpr int WSK_MAX_ROWS = 256;       // measured: beyond this the 32-row tiles re-read the operands too often and the shared-tile kernels win
static bool wsk_enabled() {
    static const bool on = std::getenv("FISE_NO_WSK") == nullptr;       // switch for A/B measurements
    return on;
}

template <int BN, int NW, int NST>
static int launch_wsk(IgemmArgs a, hipStream_t st) {
    constexpr int lds = NW * NST * (32 + BN) * 128;
    const int rows = a.B * a.Ma;
    const int ncols = a.geglu ? 2 * a.N : a.N;
    a.splits = 1; a.partial = nullptr;
    a.gx = ceil_div(rows, 32); a.gy = ceil_div(ncols, BN);
    if (a.tile_w <= 0) a.tile_w = a.tile;
    a.need_pix = a.res && a.res_compact == 0;
    for (int sct = 0; sct < a.nsect; ++sct) a.need_pix |= a.out_mode[sct] == OUT_MAP || a.out_mode[sct] == OUT_TOKENS_T;
    // raised once per instantiation (initialisation of a function-local static is thread safe)
    static const hipError_t attr = lds > 48 * 1024 ? hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_wsk_kernel<BN, NW, NST>),
                                                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds) : hipSuccess;
    if (attr != hipSuccess) return fail(FISE_ERR_HIP, "igemm: cannot raise the dynamic LDS limit");
    const double flops = 2.0 * rows * (double)ncols * (double)a.K;
    const double bytes = 2.0 * ((double)ncols * (double)a.K + (double)rows * a.C0 + (double)rows * a.N);
    {
        ProfileScope prof(PROF_IGEMM_WSK, flops, bytes, st);
        hipLaunchKernelGGL((igemm_wsk_kernel<BN, NW, NST>), dim3((unsigned)(a.gx * a.gy)), dim3(64 * NW), lds, st, a);
    }
    FISE_CHECK_LAUNCH("igemm (wave-split)");
    if (a.ln_out) {
        if (a.nsect != 1 || a.out_mode[0] != OUT_COMPACT_F32 || a.geglu || !a.ln_gamma || !a.ln_beta)
            return fail(FISE_ERR_SHAPE, "igemm: LayerNorm output needs one float compact section");
        return launch_ln_rows(a.out[0], 1, rows, a.N, a.ln_gamma, a.ln_beta, a.ln_eps, a.ln_out, nullptr, 1, 1, 1, 1, 1, st);
    }
    return FISE_OK;
}

static bool wsk_fits(const IgemmArgs& a) {
    if (!wsk_enabled()) return false;
    const int rows = a.B * a.Ma;
    if (a.pro != PRO_NONE || a.K2 != 0 || a.ksize != 1 || a.C1 != 0 || a.stride != 1 || a.ups || a.C0 % 64) return false;
    if (rows > WSK_MAX_ROWS || a.N % 4 || a.sect_n % 4) return false;
    constexpr size_t kLim = (size_t)1 << 31;            // 32-bit buffer offsets, top bit reserved for "no such row"
    const size_t npix_in = a.a_compact ? (size_t)rows : (size_t)a.B * a.Hin * a.Win;
    const size_t ncols = a.geglu ? 2 * (size_t)a.N : (size_t)a.N;
    return npix_in * a.C0 * 2 < kLim && ncols * a.K * 2 < kLim;
}

// Waves per tile (= K shares: about four K steps per wave at least) and ring depth.  Every workgroup of the launch
// should be resident at once (a second round of workgroups doubles the time of these short kernels), so the LDS a
// workgroup may take is the CU's 160 KB divided by the workgroups each of the 256 CUs has to hold.
template <int BN>
static int launch_wsk_bn(const IgemmArgs& a, hipStream_t st) {
    const int nsteps = a.K / 64;
    const int rows = a.B * a.Ma, ncols = a.geglu ? 2 * a.N : a.N;
    const int wgs = ceil_div(rows, 32) * ceil_div(ncols, BN);
    const int budget = 160 * 1024 / std::max(1, ceil_div(wgs, 256)) - 1024;
    int nw = nsteps <= 6 ? 1 : nsteps <= 12 ? 2 : 4;
    auto lds = [](int w, int n) { return w * n * (32 + BN) * 128; };
    while (nw > 1 && lds(nw, 2) > budget) nw >>= 1;
    const int nst = lds(nw, 4) <= std::min(budget, 128 * 1024) ? 4 : lds(nw, 3) <= budget ? 3 : 2;
#define FISE_WSK(W, S) if (nw == W && nst == S) return launch_wsk<BN, W, S>(a, st)
    FISE_WSK(1, 4); FISE_WSK(1, 3); FISE_WSK(1, 2);
    FISE_WSK(2, 4); FISE_WSK(2, 3); FISE_WSK(2, 2);
    FISE_WSK(4, 4); FISE_WSK(4, 3); FISE_WSK(4, 2);
#undef FISE_WSK
    return fail(FISE_ERR_SHAPE, "igemm: no wave-split configuration for %d waves, %d stages", nw, nst);
}

static int launch_wsk_any(const IgemmArgs& a, hipStream_t st) {
    return a.geglu ? launch_wsk_bn<64>(a, st) : launch_wsk_bn<32>(a, st);
}

int launch_igemm(const IgemmArgs& a, const IgemmWorkspace* ws, hipStream_t st) {
    const int rows = a.B * a.Ma;
    if (rows <= 0) return FISE_OK;
    const int Cin = a.C0 + a.C1;
    if (a.K != a.ksize * a.ksize * Cin) return fail(FISE_ERR_SHAPE, "igemm: K=%d != %d*%d*%d", a.K, a.ksize, a.ksize, Cin);
    if (a.C0 % 32 || a.C1 % 32) return fail(FISE_ERR_ALIGN, "igemm: channel counts %d,%d must be multiples of 32", a.C0, a.C1);
    if (a.a_compact && (a.ksize != 1 || a.C1 != 0)) return fail(FISE_ERR_SHAPE, "igemm: compact A needs ksize 1, one source");
    if (a.pro != PRO_NONE && (a.G < 1 || Cin % a.G)) return fail(FISE_ERR_SHAPE, "igemm: Cin=%d %% G=%d", Cin, a.G);
    if (a.nsect < 1 || a.nsect > 3 || a.nsect * a.sect_n != a.N) return fail(FISE_ERR_SHAPE, "igemm: sections");
    if (a.K2 != a.S0 + a.S1 || a.S0 % 32 || a.S1 % 32 || (a.K2 > 0 && (!a.w2 || !a.s0 || a.a_compact || a.stride != 1 || a.ups)))
        return fail(FISE_ERR_SHAPE, "igemm: side product");
    if (a.nview < 0 || a.nview > 2 || (a.nview > 0 && (a.nsect != 1 || a.out_mode[0] != OUT_MAP || a.N % 4 || a.geglu)))
        return fail(FISE_ERR_SHAPE, "igemm: normalised copies need one map section with N %% 4 == 0");
    for (int i = 0; i < a.nview; ++i)
        if (!a.view[i].dst || !a.view[i].ss || a.view[i].dstC % 4 || a.view[i].c_off % 4 || a.view[i].c_off + a.N > a.view[i].dstC)
            return fail(FISE_ERR_SHAPE, "igemm: normalised copy %d: channels %d + %d of %d", i, a.view[i].c_off, a.N, a.view[i].dstC);
    if (wsk_fits(a)) return launch_wsk_any(a, st);
    const bool wide = rows >= 4096 && a.N >= 128;          // dense-sized problems: 64x128 tiles, 8 waves
    if (a.geglu) {
        if (rows <= 32) return launch_cfg<32, 256, 1, 4>(a, ws, PROF_IGEMM_GEGLU, st);
        return launch_cfg<64, 128, 2, 2>(a, ws, PROF_IGEMM_GEGLU, st);
    }
    if (wide) return launch_cfg<64, 128, 2, 4>(a, ws, PROF_IGEMM_WIDE, st);
    if (rows <= 32) return launch_cfg<32, 128, 1, 4>(a, ws, PROF_IGEMM_THIN, st);
    return launch_cfg<64, 64, 2, 2>(a, ws, PROF_IGEMM, st);
}

}  // namespace fise

