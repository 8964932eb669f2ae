// Active-query attention on bf16 MFMA: each wave owns 32 gathered queries of one
// (batch, head) and streams keys in blocks of 64 through LDS with an online
// softmax.  Scores are computed transposed (S^T = K Q^T) so that a lane keeps one
// query's running max / sum to itself, and the output is accumulated transposed
// (O^T = V^T P^T), which is why V operands are stored keys-innermost.
//
// With few active queries there are few (query tile, head, batch) workgroups, so
// the key range is also split over workgroups: each writes an unnormalised partial
// (running max, sum, output) and a second small kernel merges the partials in
// split order.  The next key block is fetched into registers while the current
// one is being multiplied; the LDS hand-over uses a barrier that does not wait for
// those loads.
#include <algorithm>
#include "igemm.h"
#include "profile.h"

namespace fise {

constexpr int AT_BKV = 64;        // keys per block
constexpr int AT_QW = 32;         // queries per wave
constexpr int AT_WAVES = 4;
constexpr int AT_BQ = AT_QW * AT_WAVES;

__device__ __forceinline__ void at_lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int KD, int DB>          // KD: 16-wide steps over the head dim; DB: 32-row blocks of the output head dim
__global__ __launch_bounds__(256) void attention_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ K,
                                                        const bf16_t* __restrict__ Vt, int B, int M, int n_keys, int n_stride,
                                                        int C, int d, float scale_log2e, int splits, int nqt, int heads,
                                                        bf16_t* __restrict__ out, float* __restrict__ part_o, float* __restrict__ part_ml) {
    constexpr int DP = KD * 16;
    constexpr int KP = DP + 8;            // K tile pitch (bf16)
    constexpr int VP = AT_BKV + 8;        // V^T tile pitch
    constexpr int KCH = AT_BKV * (DP / 8);        // 16-byte chunks of the K tile
    constexpr int VCH = DB * 32 * (AT_BKV / 8);   // and of the V^T tile
    constexpr int KL = (KCH + 255) / 256, VL = (VCH + 255) / 256;
    __shared__ __attribute__((aligned(16))) bf16_t Ks[AT_BKV][KP];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[DB * 32][VP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hl = lane >> 5, l32 = lane & 31;
    // Workgroup -> (query tile qt, head h, batch element b, key split sp).  The grid is one-dimensional
    // and consecutive workgroups go round-robin to the 8 XCDs (one L2 each): workgroup w takes position
    // (w % 8) * (total / 8) + w / 8 of the (b, sp, h, qt) order, qt fastest, so the query tiles that
    // stream the same K / V slice run on one XCD and the slice is fetched from HBM once, not eight times.
    int qt, h, b, sp;
    {
        const int total = nqt * heads * B * splits, chunk = total >> 3;
        int w = blockIdx.x;
        if (w < (chunk << 3)) w = (w & 7) * chunk + (w >> 3);
        qt = w % nqt; int t = w / nqt;
        h = t % heads; t /= heads;
        sp = t % splits; b = t / splits;
    }
    const int qrow = qt * AT_BQ + wave * AT_QW + l32;
    const bool qok = qrow < M;
    const int dchunks = d / 8;

    // key blocks of this split
    const int nblocks = (n_keys + AT_BKV - 1) / AT_BKV;
    const int per = (nblocks + splits - 1) / splits;
    const int blk0 = sp * per, blk1 = min(nblocks, blk0 + per);

    // query fragments: B operand of S^T = K Q^T (column = query, 8 consecutive head-dim elements)
    bf16x8_t qf[KD];
#pragma unroll
    for (int ks = 0; ks < KD; ++ks) {
        const int c = ks * 16 + hl * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qok && c < d) v = *reinterpret_cast<const uint4*>(q + ((size_t)b * M + qrow) * C + h * d + c);
        qf[ks] = *reinterpret_cast<bf16x8_t*>(&v);
    }

    f32x16_t oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // ---- register staging of key blocks.  Thread slot j covers chunk e = tid + 256 j of the block's real data:
    // K rows of d / 8 chunks (key e / dchunks, chunk e % dchunks), V^T rows of 8 chunks (row e / 8 < d, keys
    // (e % 8) * 8 ..).  Everything that depends only on the slot is worked out once; a block costs one pointer
    // bump and one load per slot.  The padding of the LDS tiles (head-dim columns / rows past d) is zeroed once
    // and never written again.  Keys that do not exist can only occur in the last block of the whole range: that
    // block alone takes the guarded path (keys past n_keys read nothing and are stored as zeros).
    constexpr int PFD = (KL + VL <= 6) ? 2 : 1;       // key blocks in flight (small heads can afford two in registers)
    uint4 rk[PFD][KL], rv[PFD][VL];
    const bf16_t* pk[KL]; const bf16_t* pv[VL];        // source of the slot in key block 0
    int kkey[KL], vkey[VL];                            // first key of the slot within a block (-1: slot unused)
    bf16_t* sk[KL]; bf16_t* sv[VL];                    // destination in the LDS tiles
#pragma unroll
    for (int j = 0; j < KL; ++j) {
        const int e = tid + 256 * j;
        const int kk = e / dchunks, c8 = e - kk * dchunks;
        const bool used = e < AT_BKV * dchunks;
        kkey[j] = used ? kk : -1;
        pk[j] = K + (used ? ((size_t)b * n_keys + kk) * C + h * d + c8 * 8 : 0);
        sk[j] = &Ks[used ? kk : 0][used ? c8 * 8 : 0];
    }
#pragma unroll
    for (int j = 0; j < VL; ++j) {
        const int e = tid + 256 * j;
        const int r = e >> 3, c8 = e & 7;
        const bool used = r < d;
        vkey[j] = used ? c8 * 8 : -1;
        pv[j] = Vt + (used ? ((size_t)b * C + h * d + r) * n_stride + c8 * 8 : 0);
        sv[j] = &Vs[used ? r : 0][used ? c8 * 8 : 0];
    }
    for (int e = tid; e < AT_BKV * KP / 8; e += 256) reinterpret_cast<uint4*>(&Ks[0][0])[e] = make_uint4(0, 0, 0, 0);
    for (int e = tid; e < DB * 32 * VP / 8; e += 256) reinterpret_cast<uint4*>(&Vs[0][0])[e] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    // The query fragments must have ARRIVED before the key loop is entered: while their loads are still counted as
    // outstanding at the loop head, the compiler's wait-count bookkeeping (merged over the loop's paths) puts a
    // wait for ALL loads in front of the first MFMA of every iteration, i.e. right behind the prefetch of the next
    // key block, which then never overlaps anything.  Naming the fragments as operands here places that wait once.
#pragma unroll
    for (int ks = 0; ks < KD; ++ks) asm volatile("" ::"v"(qf[ks]));
    auto fetch = [&](int blk, int slot) {
        const int k0 = blk * AT_BKV;
        if (k0 + AT_BKV <= n_keys) {                     // uniform: a block of existing keys
#pragma unroll
            for (int j = 0; j < KL; ++j) rk[slot][j] = *reinterpret_cast<const uint4*>(pk[j] + (size_t)k0 * C);
#pragma unroll
            for (int j = 0; j < VL; ++j) rv[slot][j] = *reinterpret_cast<const uint4*>(pv[j] + k0);
        } else {
#pragma unroll
            for (int j = 0; j < KL; ++j) {
                const bool ok = kkey[j] >= 0 && k0 + kkey[j] < n_keys;
                rk[slot][j] = ok ? *reinterpret_cast<const uint4*>(pk[j] + (size_t)k0 * C) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < VL; ++j) {
                const int key = k0 + vkey[j];
                uint4 v = make_uint4(0, 0, 0, 0);
                if (vkey[j] >= 0 && key < n_keys) {
                    v = *reinterpret_cast<const uint4*>(pv[j] + k0);
                    const int nvalid = n_keys - key;          // keys of this chunk that exist; the rest become zeros
                    if (nvalid < 8) {
                        unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int t = 0; t < 8; ++t)
                            if (t >= nvalid) w4[t >> 1] &= (t & 1) ? 0x0000ffffu : 0xffff0000u;
                        v = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                    }
                }
                rv[slot][j] = v;
            }
        }
    };
    auto stash = [&](int slot) {
#pragma unroll
        for (int j = 0; j < KL; ++j)
            if (kkey[j] >= 0) *reinterpret_cast<uint4*>(sk[j]) = rk[slot][j];
#pragma unroll
        for (int j = 0; j < VL; ++j)
            if (vkey[j] >= 0) *reinterpret_cast<uint4*>(sv[j]) = rv[slot][j];
    };

    if (blk0 < blk1) {
#pragma unroll
        for (int s = 0; s < PFD; ++s) fetch(min(blk0 + s, blk1 - 1), s);
    }
    for (int blk0u = blk0; blk0u < blk1; blk0u += PFD) {
#pragma unroll
      for (int slot = 0; slot < PFD; ++slot) {
        const int blk = blk0u + slot;
        if (blk >= blk1) break;                            // uniform across the workgroup
        const int k0 = blk * AT_BKV;
        at_lds_barrier();                                  // previous block fully consumed
        stash(slot);
        fetch(min(blk + PFD, blk1 - 1), slot);             // PFD blocks ahead, in flight during the MFMAs below
        at_lds_barrier();

        // ---- S^T = K Q^T for two 32-key blocks
        f32x16_t s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KD; ++ks) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(&Ks[kb * 32 + l32][ks * 16 + hl * 8]);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
            }
        }
        // ---- online softmax (this lane: query l32; keys kb*32 + (e/4)*8 + hl*4 + e%4).  The scale is positive,
        // so the running maximum is taken over the raw scores and the scale rides on the exponent's
        // multiply-add; keys that do not exist can only be in the last block of the range.
        if (__builtin_amdgcn_readfirstlane(k0 + AT_BKV > n_keys)) {      // scalar condition: a real branch, not 32 selects
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (k0 + kb * 32 + (e >> 2) * 8 + hl * 4 + (e & 3) >= n_keys) s[kb][e] = -INFINITY;
        }
        float mraw = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mraw = fmaxf(mraw, s[kb][e]);
        mraw = fmaxf(mraw, __shfl_xor(mraw, 32));
        const float mx = fmaxf(m_run, mraw * scale_log2e);
        const float alpha = __builtin_amdgcn_exp2f(m_run - mx);   // first block: exp2(-inf) = 0
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][e], scale_log2e, -mx));   // v_exp_f32: results below 2^-126 flush to 0
                s[kb][e] = p;
                psum += p;
            }
        psum += __shfl_xor(psum, 32);
        l_run = l_run * alpha + psum;
        m_run = mx;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;

        // ---- O^T += V^T P^T : four 16-key steps; the key order inside a step follows the accumulator layout
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                uint4 pw;                                  // eight probabilities as packed bf16 pairs
                pw.x = f2bf2(s[kb][8 * jj + 0], s[kb][8 * jj + 1]); pw.y = f2bf2(s[kb][8 * jj + 2], s[kb][8 * jj + 3]);
                pw.z = f2bf2(s[kb][8 * jj + 4], s[kb][8 * jj + 5]); pw.w = f2bf2(s[kb][8 * jj + 6], s[kb][8 * jj + 7]);
                const bf16x8_t pf = *reinterpret_cast<bf16x8_t*>(&pw);
                const int kbase = kb * 32 + 16 * jj + hl * 4;
#pragma unroll
                for (int i = 0; i < DB; ++i) {
                    const uint2 lo = *reinterpret_cast<const uint2*>(&Vs[i * 32 + l32][kbase]);
                    const uint2 hi = *reinterpret_cast<const uint2*>(&Vs[i * 32 + l32][kbase + 8]);
                    uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
                    oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8_t*>(&v), pf, oacc[i], 0, 0, 0);
                }
            }
      }
    }

    // ---- store: lane holds query l32, head-dim rows i*32 + (e/4)*8 + hl*4 + e%4: four consecutive elements of e are
    // four consecutive channels (d is a multiple of 8, so a group of four is inside the head or outside it as a whole)
    if (!qok) return;
    if (splits == 1) {
        const float inv = 1.0f / l_run;
        bf16_t* o = out + ((size_t)b * M + qrow) * C + h * d;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int r = i * 32 + q4 * 8 + hl * 4;
                if (r < d)
                    *reinterpret_cast<uint2*>(o + r) = make_uint2(f2bf2(oacc[i][4 * q4] * inv, oacc[i][4 * q4 + 1] * inv),
                                                                  f2bf2(oacc[i][4 * q4 + 2] * inv, oacc[i][4 * q4 + 3] * inv));
            }
    } else {
        // unnormalised partial of this key range: O[sp][b][qrow][h*d + r], (m, l)[sp][b][h][qrow]
        float* po = part_o + (((size_t)sp * B + b) * M + qrow) * C + h * d;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int r = i * 32 + q4 * 8 + hl * 4;
                if (r < d)
                    *reinterpret_cast<float4*>(po + r) = make_float4(oacc[i][4 * q4], oacc[i][4 * q4 + 1], oacc[i][4 * q4 + 2], oacc[i][4 * q4 + 3]);
            }
        if (hl == 0) {
            float* pm = part_ml + ((((size_t)sp * B + b) * heads + h) * M + qrow) * 2;
            pm[0] = m_run; pm[1] = l_run;
        }
    }
}

// out[b,m,c] = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^(m_s - max_s m_s), splits visited in index order.
// One thread per four channels (d is a multiple of 8: the four share a head, hence the weights).
__global__ __launch_bounds__(256) void attention_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                              int B, int M, int C, int heads, int d, int splits,
                                                              bf16_t* __restrict__ out) {
    const int C4 = C / 4;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)B * M * C4) return;
    const int c = (int)(i % C4) * 4, m = (int)((i / C4) % M), b = (int)(i / ((long long)C4 * M));
    const int h = c / d;
    const size_t ml_stride = (size_t)B * heads * M * 2, o_stride = (size_t)B * M * C;
    const float* ml0 = part_ml + (((size_t)b * heads + h) * M + m) * 2;
    const float* o0 = part_o + ((size_t)b * M + m) * C + c;
    float mx = -INFINITY;
#pragma unroll 8
    for (int s = 0; s < splits; ++s) mx = fmaxf(mx, ml0[s * ml_stride]);     // unrolled: the loads go out together, not one round trip each
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    float den = 0.f;
#pragma unroll 4
    for (int s = 0; s < splits; ++s) {
        const float2 ml = *reinterpret_cast<const float2*>(ml0 + s * ml_stride);
        const float4 o = *reinterpret_cast<const float4*>(o0 + s * o_stride);
        const float w = __builtin_amdgcn_exp2f(ml.x - mx);  // an empty split has m = -inf: weight 0
        num.x += w * o.x; num.y += w * o.y; num.z += w * o.z; num.w += w * o.w;
        den += w * ml.y;
    }
    const float inv = 1.0f / den;
    *reinterpret_cast<uint2*>(out + ((size_t)b * M + m) * C + c) = make_uint2(f2bf2(num.x * inv, num.y * inv), f2bf2(num.z * inv, num.w * inv));
}

template <int KD, int DB>
static void launch_at(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C, int heads,
                      int d, float scale, int splits, void* out, float* part_o, float* part_ml, hipStream_t st) {
    const int nqt = ceil_div(M, AT_BQ);
    dim3 grid((unsigned)(nqt * heads * B * splits));
    hipLaunchKernelGGL((attention_kernel<KD, DB>), grid, dim3(256), 0, st, (const bf16_t*)q, (const bf16_t*)K,
                       (const bf16_t*)Vt, B, M, n_keys, n_stride, C, d, scale * 1.4426950408889634f, splits, nqt, heads,
                       (bf16_t*)out, part_o, part_ml);
}

static int attention_splits(int B, int M, int n_keys, int heads) {
    const int wgs = ceil_div(M, AT_BQ) * heads * B;
    const int nblocks = ceil_div(n_keys, AT_BKV);
    int s = ceil_div(640, wgs);
    s = std::min(s, nblocks / 2);
    return std::max(1, std::min(s, 32));
}

size_t attention_workspace_bytes(int B, int M, int n_keys, int C, int heads) {
    const int s = attention_splits(B, M, n_keys, heads);
    if (s <= 1) return 0;
    return align256((size_t)s * B * M * C * sizeof(float)) + align256((size_t)s * B * heads * M * 2 * sizeof(float));
}

int launch_attention(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C, int heads,
                     float scale, void* out, void* ws, size_t ws_bytes, hipStream_t st) {
    if (M <= 0) return FISE_OK;
    const int d = C / heads;
    const int kd = ceil_div(d, 16), db = ceil_div(d, 32);
    int splits = attention_splits(B, M, n_keys, heads);
    if (splits > 1 && (!ws || ws_bytes < attention_workspace_bytes(B, M, n_keys, C, heads))) splits = 1;
    float* part_o = (float*)ws;
    float* part_ml = splits > 1 ? (float*)((char*)ws + align256((size_t)splits * B * M * C * sizeof(float))) : nullptr;
    {
    ProfileScope prof(PROF_ATTENTION, 4.0 * B * (double)M * n_keys * C,
                      2.0 * ((double)B * n_keys * C * 2 + 2.0 * B * M * C), st);
#define FISE_AT(KDV, DBV) launch_at<KDV, DBV>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, splits, out, part_o, part_ml, st)
    if (kd <= 1) FISE_AT(1, 1);
    else if (kd == 2) FISE_AT(2, 1);
    else if (kd == 3) FISE_AT(3, 2);
    else if (kd == 4) FISE_AT(4, 2);
    else if (kd <= 6 && db <= 3) FISE_AT(6, 3);
    else if (kd <= 8) FISE_AT(8, 4);
    else if (kd <= 10) FISE_AT(10, 5);
    else return fail(FISE_ERR_SHAPE, "attention: head dim %d > 160", d);
#undef FISE_AT
    }
    FISE_CHECK_LAUNCH("attention");
    if (splits > 1) {
        const long long n = (long long)B * M * (C / 4);
        ProfileScope prof(PROF_ATTENTION_MERGE, 0.0, (double)splits * B * M * C * 4.0 + 2.0 * B * M * C, st);
        hipLaunchKernelGGL(attention_merge_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part_o, part_ml, B, M, C,
                           heads, d, splits, (bf16_t*)out);
        FISE_CHECK_LAUNCH("attention merge");
    }
    return FISE_OK;
}

}  // namespace fise

using namespace fise;

extern "C" size_t fise_attention_active_workspace_bytes(int B, int M, int n_keys, int C, int heads) {
    if (B < 1 || M < 1 || n_keys < 1 || C < 1 || heads < 1) return 0;
    return attention_workspace_bytes(B, M, n_keys, C, heads);
}

extern "C" int fise_attention_active(const void* q, const void* K, const void* Vt, int dtype, int B, int M, int n_keys,
                                     int n_stride, int C, int heads, float scale, void* out, void* workspace,
                                     size_t workspace_bytes, void* stream) {
    if (!q || !K || !Vt || !out) return fail(FISE_ERR_NULL, "fise_attention_active: null pointer");
    if (dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_attention_active: bf16 only (dtype %d)", dtype);
    if (B < 1 || M < 0 || n_keys < 1 || C < 1 || heads < 1 || C % heads) return fail(FISE_ERR_SHAPE, "fise_attention_active: B%d M%d keys%d C%d heads%d", B, M, n_keys, C, heads);
    const int d = C / heads;
    if (d % 8 || d > 160) return fail(FISE_ERR_SHAPE, "fise_attention_active: head dim %d (multiple of 8, <= 160)", d);
    if (n_stride < n_keys || n_stride % 8) return fail(FISE_ERR_ALIGN, "fise_attention_active: n_stride %d (>= n_keys, multiple of 8)", n_stride);
    if (!aligned16(q) || !aligned16(K) || !aligned16(Vt) || !aligned16(out) || (workspace && !aligned16(workspace)))
        return fail(FISE_ERR_ALIGN, "fise_attention_active: pointers must be 16-byte aligned");
    return launch_attention(q, K, Vt, B, M, n_keys, n_stride, C, heads, scale, out, workspace, workspace_bytes, as_stream(stream));
}
