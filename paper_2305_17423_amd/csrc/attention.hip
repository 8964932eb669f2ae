// Active-query attention on bf16 MFMA: each wave owns 32 gathered queries of one
// (batch, head) and streams all keys in blocks of 64 through LDS with an online
// softmax.  Scores are computed transposed (S^T = K Q^T) so that a lane keeps one
// query's running max / sum to itself, and the output is accumulated transposed
// (O^T = V^T P^T), which is why V operands are stored keys-innermost.
#include "igemm.h"
#include "profile.h"

namespace fise {

constexpr int AT_BKV = 64;        // keys per block
constexpr int AT_QW = 32;         // queries per wave
constexpr int AT_WAVES = 4;

template <int KD, int DB>          // KD: 16-wide steps over the head dim; DB: 32-row blocks of the output head dim
__global__ __launch_bounds__(256) void attention_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ K,
                                                        const bf16_t* __restrict__ Vt, int M, int n_keys, int n_stride,
                                                        int C, int d, float scale_log2e, bf16_t* __restrict__ out) {
    constexpr int DP = KD * 16;
    constexpr int KP = DP + 8;            // K tile pitch (bf16)
    constexpr int VP = AT_BKV + 8;        // V^T tile pitch
    __shared__ __attribute__((aligned(16))) bf16_t Ks[AT_BKV][KP];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[DB * 32][VP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hl = lane >> 5, l32 = lane & 31;
    const int h = blockIdx.y, b = blockIdx.z;
    const int qrow = blockIdx.x * (AT_QW * AT_WAVES) + wave * AT_QW + l32;
    const bool qok = qrow < M;

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

    const int dchunks = d / 8;
    for (int k0 = 0; k0 < n_keys; k0 += AT_BKV) {
        __syncthreads();                                   // previous block fully consumed
        // ---- K tile: [64 keys][DP], zero padded
        for (int e = tid; e < AT_BKV * (DP / 8); e += 256) {
            const int kk = e / (DP / 8), c8 = e % (DP / 8);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (k0 + kk < n_keys && c8 < dchunks)
                v = *reinterpret_cast<const uint4*>(K + ((size_t)b * n_keys + k0 + kk) * C + h * d + c8 * 8);
            *reinterpret_cast<uint4*>(&Ks[kk][c8 * 8]) = v;
        }
        // ---- V^T tile: [DB*32 head-dim rows][64 keys], zero where the row or the key does not exist
        for (int e = tid; e < DB * 32 * (AT_BKV / 8); e += 256) {
            const int r = e / (AT_BKV / 8), c8 = e % (AT_BKV / 8);
            const int key = k0 + c8 * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r < d && key < n_keys) {
                v = *reinterpret_cast<const uint4*>(Vt + ((size_t)b * C + h * d + r) * n_stride + key);
                const int nvalid = n_keys - key;           // >= 1
                if (nvalid < 8) {
                    unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (j >= nvalid) w4[j >> 1] &= (j & 1) ? 0x0000ffffu : 0xffff0000u;
                    v = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                }
            }
            *reinterpret_cast<uint4*>(&Vs[r][c8 * 8]) = v;
        }
        __syncthreads();

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
        // ---- online softmax (this lane: query l32; keys kb*32 + (e/4)*8 + hl*4 + e%4)
        float mx = m_run;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = k0 + kb * 32 + (e >> 2) * 8 + hl * 4 + (e & 3);
                const float v = key < n_keys ? s[kb][e] * scale_log2e : -INFINITY;
                s[kb][e] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float alpha = exp2f(m_run - mx);            // first block: exp2(-inf) = 0
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = exp2f(s[kb][e] - mx);
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
                bf16x8_t pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (short)f2bf(s[kb][8 * jj + e]);
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

    // ---- normalise and store: lane holds query l32, head-dim rows i*32 + (e/4)*8 + hl*4 + e%4
    if (qok) {
        const float inv = 1.0f / l_run;
        bf16_t* o = out + ((size_t)b * M + qrow) * C + h * d;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = i * 32 + (e >> 2) * 8 + hl * 4 + (e & 3);
                if (r < d) o[r] = f2bf(oacc[i][e] * inv);
            }
    }
}

template <int KD, int DB>
static void launch_at(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C, int heads,
                      int d, float scale, void* out, hipStream_t st) {
    dim3 grid(ceil_div(M, AT_QW * AT_WAVES), heads, B);
    hipLaunchKernelGGL((attention_kernel<KD, DB>), grid, dim3(256), 0, st, (const bf16_t*)q, (const bf16_t*)K,
                       (const bf16_t*)Vt, M, n_keys, n_stride, C, d, scale * 1.4426950408889634f, (bf16_t*)out);
}

int launch_attention(const void* q, const void* K, const void* Vt, int B, int M, int n_keys, int n_stride, int C, int heads,
                     float scale, void* out, hipStream_t st) {
    if (M <= 0) return FISE_OK;
    const int d = C / heads;
    const int kd = ceil_div(d, 16), db = ceil_div(d, 32);
    ProfileScope prof(PROF_ATTENTION, 4.0 * B * (double)M * n_keys * C,
                      2.0 * ((double)B * n_keys * C * 2 + 2.0 * B * M * C), st);
    if (kd <= 1) launch_at<1, 1>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else if (kd == 2) launch_at<2, 1>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else if (kd == 3) launch_at<3, 2>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else if (kd == 4) launch_at<4, 2>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else if (kd <= 6 && db <= 3) launch_at<6, 3>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else if (kd <= 8) launch_at<8, 4>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else if (kd <= 10) launch_at<10, 5>(q, K, Vt, B, M, n_keys, n_stride, C, heads, d, scale, out, st);
    else return fail(FISE_ERR_SHAPE, "attention: head dim %d > 160", d);
    FISE_CHECK_LAUNCH("attention");
    return FISE_OK;
}

}  // namespace fise

using namespace fise;

extern "C" int fise_attention_active(const void* q, const void* K, const void* Vt, int dtype, int B, int M, int n_keys,
                                     int n_stride, int C, int heads, float scale, void* out, void* stream) {
    if (!q || !K || !Vt || !out) return fail(FISE_ERR_NULL, "fise_attention_active: null pointer");
    if (dtype != FISE_BF16) return fail(FISE_ERR_DTYPE, "fise_attention_active: bf16 only (dtype %d)", dtype);
    if (B < 1 || M < 0 || n_keys < 1 || C < 1 || heads < 1 || C % heads) return fail(FISE_ERR_SHAPE, "fise_attention_active: B%d M%d keys%d C%d heads%d", B, M, n_keys, C, heads);
    const int d = C / heads;
    if (d % 8 || d > 160) return fail(FISE_ERR_SHAPE, "fise_attention_active: head dim %d (multiple of 8, <= 160)", d);
    if (n_stride < n_keys || n_stride % 8) return fail(FISE_ERR_ALIGN, "fise_attention_active: n_stride %d (>= n_keys, multiple of 8)", n_stride);
    if (!aligned16(q) || !aligned16(K) || !aligned16(Vt) || !aligned16(out)) return fail(FISE_ERR_ALIGN, "fise_attention_active: pointers must be 16-byte aligned");
    return launch_attention(q, K, Vt, B, M, n_keys, n_stride, C, heads, scale, out, as_stream(stream));
}
