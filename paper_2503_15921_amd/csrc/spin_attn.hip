// Attention kernels of the verification step for gfx950 (CDNA4, 64-wide wavefronts).
//
// Computes Eq. (2) of Sec. II-A1 for the draft rows of every request over the keys they may
// see, read through a page table; pieces of one request are rejoined with the single
// denominator of Eq. (13), Sec. V-A.
//
// One wavefront works on one item = (draft rows x query heads of one KV group) x (a run of
// keys) of one request and one KV head.  It streams the K and V rows of 32 keys at a time:
//   * K: every lane fetches 16 contiguous bytes so that one load instruction covers 1 KiB of
//     contiguous cache, the tile is re-shaped through LDS (padded rows, conflict-free) into the
//     MFMA operand layout [key][32 head dims], and S^T = K Q^T is formed with
//     v_mfma_f32_16x16x32_bf16 -- the keys on the 16-row side, the (few, ragged) query rows on
//     the 16-column side, so row padding wastes matrix-core columns, never memory traffic.
//   * softmax: each query row lives in four lanes; running maximum and sum are kept online,
//     the maximum is exchanged with two wavefront shuffles per block.
//   * V: O^T = V^T P^T.  The contraction runs over keys, so the operand needs, per lane, eight
//     keys of one head dim.  Each lane fetches the same 16-byte column chunk of eight keys
//     (256 contiguous bytes per key row across 16 lanes) and transposes the 8x8 block of
//     16-bit values in registers with byte permutes; V never touches LDS.  The key order of the
//     contraction is chosen to be the order in which the score tile already holds P, so P goes
//     from accumulator to operand without leaving its lane.
// The next block's K and V are in flight (in registers) while the current one is consumed.
// Un-normalised results (running max, sum, O) go to a partial buffer; a second kernel joins the
// partials of each (row, head) and writes bf16.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spin_device.h"

namespace spin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kNegBig = -1.0e30f;   // running-max start: finite, so (m_old - m_new) is never NaN

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 v = {(__bf16)lo, (__bf16)hi};   // round to nearest even
    return __builtin_bit_cast(uint32_t, v);
}

// K/V bytes are used once: a non-temporal load keeps them from displacing anything in the caches
// and streams measurably faster from HBM on this part.
__device__ __forceinline__ u32x4 stream_load(const uint16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

template <int D, int NT>
__global__ __launch_bounds__(64) void verify_attn_kernel(AttnParams P) {
    constexpr int DCH = D / 8;      // 16-byte chunks per key row
    constexpr int KCALLS = D / 32;  // MFMA calls (32 head dims each) per 16-key score tile
    constexpr int KLOADS = DCH / 2; // 16-byte loads per lane for 32 keys of K
    constexpr int LROW = D + 8;     // LDS row pitch in elements: 16 bytes of padding per key
    __shared__ __attribute__((aligned(16))) uint16_t sK[32 * LROW];
    __shared__ int32_t sPT[kMaxItemPages];

    const int lane = threadIdx.x;
    const int m16 = lane & 15, g = lane >> 4;
    const int n_kv = P.n_kv_heads;
    const int kvh = blockIdx.x % n_kv;
    const Item it = P.items[P.order[blockIdx.x / n_kv]];
    const int G = P.group;
    const int pshift = P.page_shift;
    const int pmask = (1 << pshift) - 1;
    const int k0 = it.k0, k1 = it.k1;

    // page ids of this item
    const int pg0 = k0 >> pshift;
    const int npg = ((k1 - 1) >> pshift) - pg0 + 1;
    for (int i = lane; i < npg; i += 64) sPT[i] = P.page_table[it.pt_base + pg0 + i];

    // query operands and per-row visibility limits
    bf16x8 qf[NT][KCALLS];
    int lim[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int nn = nt * 16 + m16;
        const int tl = nn / G, hg = nn - tl * G;
        const bool valid = tl < it.n_q;
        lim[nt] = valid ? min(k1, it.causal0 + tl) : k0;
        const uint16_t* qp = P.q + ((int64_t)(it.q_row0 + (valid ? tl : 0)) * P.n_q_heads + kvh * G + hg) * D + g * 8;
#pragma unroll
        for (int c = 0; c < KCALLS; ++c) {
            u32x4 v = valid ? *(const u32x4*)(qp + c * 32) : u32x4{0, 0, 0, 0};
            qf[nt][c] = __builtin_bit_cast(bf16x8, v);
        }
    }
    __syncthreads();

    const int64_t head_off = (int64_t)kvh * P.head_stride;
    auto row_ptr = [&](const uint16_t* pool, int key) -> const uint16_t* {
        key = min(key, k1 - 1);   // keys past the item's end are masked; fetch a valid row instead
        const int pg = sPT[(key >> pshift) - pg0];
        return pool + (int64_t)pg * P.page_stride + head_off + (int64_t)(key & pmask) * P.token_stride;
    };
    u32x4 Kr[KLOADS], Vr[8];
    auto load_k = [&](int kb) {
#pragma unroll
        for (int i = 0; i < KLOADS; ++i) {
            const int f = i * 64 + lane;
            Kr[i] = stream_load(row_ptr(P.k_pool, kb + f / DCH) + (f % DCH) * 8);
        }
    };
    auto load_v = [&](int kb) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int kl = (j >> 2) * 16 + g * 4 + (j & 3);
            Vr[j] = stream_load(row_ptr(P.v_pool, kb + kl) + (m16 % DCH) * 8);
        }
    };

    f32x4 O[NT][8];
    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = kNegBig;
        l_run[nt] = 0.f;
#pragma unroll
        for (int jd = 0; jd < 8; ++jd) O[nt][jd] = f32x4{0, 0, 0, 0};
    }

    const int full_end = min(k1, it.causal0);   // keys below this are visible to every row of the item
    load_k(k0);
    load_v(k0);
    for (int kb = k0; kb < k1; kb += 32) {
        // ---- K: registers -> LDS in operand shape
        __syncthreads();
#pragma unroll
        for (int i = 0; i < KLOADS; ++i) {
            const int f = i * 64 + lane;
            *(u32x4*)&sK[(f / DCH) * LROW + (f % DCH) * 8] = Kr[i];
        }
        __syncthreads();
        load_k(kb + 32);   // past the item's end this re-reads its last key row (clamped): harmless

        // ---- S^T = K Q^T
        f32x4 S[2][NT];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) S[t][nt] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < KCALLS; ++c) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)&sK[(t * 16 + m16) * LROW + (c * 4 + g) * 8]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    S[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[nt][c], S[t][nt], 0, 0, 0);
            }

        // ---- online softmax; lane (row, g) holds keys kb + t*16 + g*4 + r
        const bool full = kb + 32 <= full_end;
        bf16x8 Pb[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float s[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] = S[e >> 2][nt][e & 3];
            if (!full) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = kb + (e >> 2) * 16 + g * 4 + (e & 3);
                    if (key >= lim[nt]) s[e] = -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[nt], mx * P.scale_log2);
            const float alpha = fast_exp2(m_run[nt] - m_new);
            m_run[nt] = m_new;
            float p[8], sum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                p[e] = fast_exp2(s[e] * P.scale_log2 - m_new);
                sum += p[e];
            }
            l_run[nt] = l_run[nt] * alpha + sum;
#pragma unroll
            for (int jd = 0; jd < 8; ++jd) O[nt][jd] *= alpha;
            u32x4 pk = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
            Pb[nt] = __builtin_bit_cast(bf16x8, pk);
        }

        // ---- V: 8x8 transpose of 16-bit values inside each lane, then O^T += V^T P^T
        u32x4 Vt[8];
#pragma unroll
        for (int jd = 0; jd < 8; ++jd) {
            const uint32_t sel = (jd & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
            for (int kp = 0; kp < 4; ++kp)
                Vt[jd][kp] = __builtin_amdgcn_perm(Vr[2 * kp + 1][jd >> 1], Vr[2 * kp][jd >> 1], sel);
        }
        load_v(kb + 32);
#pragma unroll
        for (int jd = 0; jd < 8; ++jd) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, Vt[jd]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                O[nt][jd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, Pb[nt], O[nt][jd], 0, 0, 0);
        }
    }

    // ---- partial result: lane (row, g) holds, per jd, head dims (g*4 + r)*8 + jd, r = 0..3.
    // Stored as [jd][16] so that each lane writes 16 contiguous bytes; the join kernel undoes it.
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float l = l_run[nt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int nn = nt * 16 + m16;
        const int tl = nn / G;
        if (tl < it.n_q) {
            const int64_t slot = (int64_t)it.part_base + (int64_t)kvh * (it.n_q * G) + nn;
            float* po = P.part_o + slot * kPartRow;
            if (g * 4 < DCH) {
#pragma unroll
                for (int jd = 0; jd < 8; ++jd) *(f32x4*)(po + jd * 16 + g * 4) = O[nt][jd];
            }
            if (g == 0) {
                P.part_ml[slot * 2] = m_run[nt];
                P.part_ml[slot * 2 + 1] = l;
            }
        }
    }
}

// Join the pieces of one (packed row, query head): Eq. (13) -- one denominator over all tokens
// of the original request.  With piece s holding (m_s, l_s, N_s) where l_s = sum of exp2(score -
// m_s) and N_s the matching weighted value sum:  O = sum_s 2^(m_s-M) N_s / sum_s 2^(m_s-M) l_s.
// One wavefront per (row, head); lane (chunk, jp) owns head dims chunk*8 + 2*jp and +1, which the
// attention kernel left at partial elements (2*jp)*16 + chunk and (2*jp+1)*16 + chunk.
constexpr int kJoinWaves = 4;

template <int D>
__global__ __launch_bounds__(64 * kJoinWaves) void join_partials_kernel(JoinParams P) {
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * kJoinWaves + (threadIdx.x >> 6);
    if (w >= (int64_t)P.n_rows * P.n_q_heads) return;
    const int r = (int)(w / P.n_q_heads), h = (int)(w - (int64_t)r * P.n_q_heads);
    const int G = P.group;
    const int kvh = h / G, hg = h - kvh * G;
    const int req = P.row_req[r];
    const int kb = P.item_begin[req], ke = P.item_begin[req + 1];
    const int chunk = lane & 15, jp = lane >> 4;
    const int e0 = (2 * jp) * 16 + chunk;
    const bool active = chunk * 8 < D;

    float M = kNegBig, den = 0.f, n0 = 0.f, n1 = 0.f;
#pragma unroll 4
    for (int k = kb; k < ke; ++k) {
        const Item it = P.items[k];
        const int tl = r - it.q_row0;
        if (tl < 0 || tl >= it.n_q) continue;
        const int64_t slot = (int64_t)it.part_base + (int64_t)kvh * (it.n_q * G) + tl * G + hg;
        const float m = P.part_ml[slot * 2], l = P.part_ml[slot * 2 + 1];
        const float o0 = P.part_o[slot * kPartRow + e0], o1 = P.part_o[slot * kPartRow + e0 + 16];
        const float Mn = fmaxf(M, m);
        const float a = fast_exp2(M - Mn), b = fast_exp2(m - Mn);
        den = den * a + l * b;
        n0 = n0 * a + o0 * b;
        n1 = n1 * a + o1 * b;
        M = Mn;
    }
    if (active) {
        const float inv = 1.0f / den;
        uint32_t* op = reinterpret_cast<uint32_t*>(P.o + ((int64_t)r * P.n_q_heads + h) * D + chunk * 8 + 2 * jp);
        *op = pack_bf16(n0 * inv, n1 * inv);
    }
}

template <int D>
static hipError_t launch_attn_d(const AttnParams& base, const int32_t* const order_dev[3], const int32_t n_in_class[3],
                                const JoinParams& jp, int n_rows, hipStream_t stream, hipEvent_t ev_mid) {
    for (int cls = 0; cls < 3; ++cls) {
        if (n_in_class[cls] == 0) continue;
        AttnParams p = base;
        p.order = order_dev[cls];
        const int64_t blocks = (int64_t)n_in_class[cls] * p.n_kv_heads;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        dim3 grid((unsigned)blocks), block(64);
        if (cls == 0) hipLaunchKernelGGL((verify_attn_kernel<D, 1>), grid, block, 0, stream, p);
        else if (cls == 1) hipLaunchKernelGGL((verify_attn_kernel<D, 2>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((verify_attn_kernel<D, 4>), grid, block, 0, stream, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (ev_mid) {
        hipError_t e = hipEventRecord(ev_mid, stream);
        if (e != hipSuccess) return e;
    }
    if (n_rows > 0) {
        const int64_t waves = (int64_t)n_rows * jp.n_q_heads;
        dim3 grid((unsigned)((waves + kJoinWaves - 1) / kJoinWaves)), block(64 * kJoinWaves);
        hipLaunchKernelGGL((join_partials_kernel<D>), grid, block, 0, stream, jp);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_attn(int head_dim, const AttnParams& base, const int32_t* const order_dev[3],
                       const int32_t n_in_class[3], const JoinParams& jp, int n_rows, hipStream_t stream,
                       hipEvent_t ev_mid) {
    if (head_dim == 128) return launch_attn_d<128>(base, order_dev, n_in_class, jp, n_rows, stream, ev_mid);
    if (head_dim == 64) return launch_attn_d<64>(base, order_dev, n_in_class, jp, n_rows, stream, ev_mid);
    return hipErrorInvalidValue;
}

}  // namespace spin
