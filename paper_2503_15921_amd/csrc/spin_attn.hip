// Attention kernels of the verification step for gfx950 (CDNA4, 64-wide wavefronts).
//
// Computes Eq. (2) of Sec. II-A1 for the draft rows of every request over the keys they may
// see, read through a page table; pieces of one request are rejoined with the single
// denominator of Eq. (13), Sec. V-A.
//
// The launch holds as many wavefronts as the chip keeps resident (one per workgroup).  The host
// has cut the sequence of all 32-key blocks of all (rectangle of draft rows x keys, KV head)
// pairs into equal shares, one per wavefront; a share is a list of pieces, each a run of blocks
// of one (rectangle, KV head).  A wavefront streams its pieces back to back:
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
//   * The block after the current one -- the next of this piece or the first of the next piece --
//     is always in flight (in registers) while the current one is consumed; descriptors and
//     page ids of later pieces are fetched pieces ahead, so the stream never drains between
//     pieces.  K/V loads are non-temporal.
//   * A (rectangle, KV head) that one wavefront held completely, and that holds every key its
//     rows may see, is normalised to bf16 at once.  Otherwise the un-normalised result (running
//     max, sum, O) goes to a partial buffer and join_partials_kernel applies Eq. (13).  Either
//     way the rows wait in LDS and are stored when the wavefront's share ends: a global store in
//     the middle of the stream would hold up the loads issued after it.
//   * Rectangles of up to 16 (draft row x query head) rows use one MFMA column tile per wavefront,
//     up to 32 rows two (verify_attn_kernel<D, 1 | 2>); wider ones, up to 64 rows, go to
//     verify_attn_group_kernel, where four wavefronts stream K/V into LDS for four that compute.
//   * TREE = true: drafts are token trees; a draft key is visible to a row only if the row's
//     ancestor mask says so (checked only in the blocks that reach into the draft region).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <algorithm>
#include <string.h>

#include "spin_device.h"

namespace spin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kNegBig = -1.0e30f;   // running-max start: finite, so (m_old - m_new) is never NaN
constexpr float kSlack = 6.0f;        // log2 of how far a score may exceed the exponent reference (grouped kernel)

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// The two 16-bit element types of Q, K, V and the output.  The kernels move elements as bit patterns
// (loads, the LDS re-shaping, the 8x8 transpose of V); only the matrix-core instruction and the
// rounding of fp32 values (P before P.V, the final rows) depend on the type.
struct Bf16 {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        bf16x2 v = {(__bf16)lo, (__bf16)hi};   // round to nearest even
        return __builtin_bit_cast(uint32_t, v);
    }
};
struct F16 {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        f16x2 v = {(_Float16)lo, (_Float16)hi};   // round to nearest even
        return __builtin_bit_cast(uint32_t, v);
    }
};

// K/V bytes are used once: a non-temporal load keeps them from displacing anything in the caches
// and streams measurably faster from HBM on this part.
__device__ __forceinline__ u32x4 stream_load(const uint16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
// the same from a wavefront-uniform base plus a 32-bit per-lane byte offset (scalar base + vector offset addressing)
__device__ __forceinline__ u32x4 stream_load(const char* base, uint32_t byte_off) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + byte_off));
}

// Where the tables of a small call sit: in the argument segment, behind the parameter block of type Params.
template <class Params>
__device__ __forceinline__ const char* inline_tables_base() {
    return (const char*)__builtin_amdgcn_kernarg_segment_ptr() + ((sizeof(Params) + 15) & ~(size_t)15);
}
template <class T>
__device__ __forceinline__ void rebase(const T*& p, const char* base) {
    p = (const T*)(base + (uintptr_t)p);
}

template <bool TREE>
__device__ __forceinline__ void use_inline_tables(AttnParams& P) {
    const char* base = inline_tables_base<AttnParams>();
    rebase(P.pieces, base);
    rebase(P.wave_begin, base);
    rebase(P.share_first, base);
    rebase(P.page_table, base);
    if (TREE) rebase(P.tree_rows, base);
}

template <int D, int NT, bool TREE, class E>
__device__ __forceinline__ void verify_attn_body(const AttnParams& P) {
    typedef typename E::vec8 vec8;
    constexpr int DCH = D / 8;      // 16-byte chunks per key row
    constexpr int KCALLS = D / 32;  // MFMA calls (32 head dims each) per 16-key score tile
    constexpr int KLOADS = DCH / 2; // 16-byte loads per lane for 32 keys of K
    constexpr int LROW = D + 8;     // LDS row pitch in elements: 16 bytes of padding per key
    constexpr int PTR = (kMaxPiecePages + 63) / 64;   // page ids per lane
    __shared__ __attribute__((aligned(16))) uint16_t sK[32 * LROW];
    __shared__ int32_t sPT[3][PTR * 64];   // page ids of the current piece and the two after it
    // Finished rows wait here until the share ends (or the space runs out) and leave together: a store
    // into global memory in the middle of the stream would hold up every load issued after it.
    // Units of 4 KiB per column tile: final rows take one ([4][64] x 16 bytes); partial rows wait as the raw
    // fp32 accumulators, two units ([8][64] x 16 bytes), and are turned into what the join kernel reads -- the
    // row normalised by its own sum, IEEE half precision whatever the element type, next to its (maximum,
    // sum) pair -- when they leave, after the wavefront's stream has ended.
    static_assert(NT <= 2, "result staging is laid out for at most two column tiles");
    constexpr int kStageUnits = 6, kStageEntries = 6;
    __shared__ u32x4 sStage[kStageUnits * 256];
    __shared__ float sStageML[kStageEntries][NT * 32];
    __shared__ int32_t sStageDesc[kStageEntries][4];   // head | flags, first row, rows, first partial slot
    int st_n = 0, st_units = 0;

    const int lane = threadIdx.x;
    const int m16 = lane & 15, g = lane >> 4;
    const int G = P.group;
    const int pshift = P.page_shift;
    const int pmask = (1 << pshift) - 1;
    // send the staged rows on their way; lane (m16, g) reads back exactly what it parked
    auto flush = [&]() {
        int unit = 0;
        for (int e = 0; e < st_n; ++e) {
            const int hf = __builtin_amdgcn_readfirstlane(sStageDesc[e][0]);
            const int q_row0 = __builtin_amdgcn_readfirstlane(sStageDesc[e][1]);
            const int n_q = __builtin_amdgcn_readfirstlane(sStageDesc[e][2]);
            const int out_base = __builtin_amdgcn_readfirstlane(sStageDesc[e][3]);
            const int kvh = hf & kPieceHeadMask;
            const bool direct = hf & kPieceDirect;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int nn = nt * 16 + m16;
                const int tl = nn / G, hg = nn - tl * G;
                const u32x4* src = sStage + unit * 256 + lane;
                if (direct) {
                    // final rows: for fixed r the eight jd are eight consecutive head dims = 16 bytes
                    if (tl < n_q && g * 4 < DCH) {
                        uint16_t* op = P.o + ((int64_t)(q_row0 + tl) * P.n_q_heads + kvh * G + hg) * D + g * 32;
#pragma unroll
                        for (int r = 0; r < 4; ++r) *(u32x4*)(op + r * 8) = src[r * 64];
                    }
                    unit += 1;
                } else {
                    if (tl < n_q) {
                        const int64_t slot = (int64_t)out_base + nn;
                        const float m = sStageML[e][nn * 2], l = sStageML[e][nn * 2 + 1];
                        const float inv = l > 0.f ? 1.0f / l : 0.f;      // (a row that saw no key: all zero, weight zero)
                        if (g * 4 < DCH) {
                            f32x4 o[8];
#pragma unroll
                            for (int jd = 0; jd < 8; ++jd) o[jd] = __builtin_bit_cast(f32x4, src[jd * 64]);
                            uint16_t* op = P.part_o + slot * kPartRow + g * 32;
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                *(u32x4*)(op + r * 8) = u32x4{F16::pack(o[0][r] * inv, o[1][r] * inv), F16::pack(o[2][r] * inv, o[3][r] * inv),
                                                              F16::pack(o[4][r] * inv, o[5][r] * inv), F16::pack(o[6][r] * inv, o[7][r] * inv)};
                        }
                        if (g == 0) {
                            P.part_ml[slot * 2] = m;
                            P.part_ml[slot * 2 + 1] = l;
                        }
                    }
                    unit += 2;
                }
            }
        }
        st_n = 0;
        st_units = 0;
    };
    // A wavefront first streams its own share, then takes queued chunks until none are left.
    for (int share = blockIdx.x;;) {
    const int pc_begin = P.wave_begin[share], pc_end = P.wave_begin[share + 1];
    if (pc_begin < pc_end) {   // (shares are never empty; an empty one would have no valid row to fetch)

    // Descriptor r of this wavefront's share (k0 == k1 when the share is exhausted).  Read through
    // the constant address space: the descriptors are never written by this kernel, which lets the
    // compiler fetch them with scalar loads.
    auto fetch_piece = [&](int r, Piece& pc) {
        if (pc_begin + r < pc_end) {
            typedef const int32_t __attribute__((address_space(4)))* ConstWords;
            const ConstWords w = (ConstWords)(uintptr_t)(P.pieces + pc_begin + r);
            pc = Piece{w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]};
        } else {
            pc = Piece{0, 0, 0, 0, 0, 0, 0, 0};
        }
    };
    auto load_pages = [&](const Piece& pc, int32_t (&pr)[PTR]) {
        const int pg0 = pc.k0 >> pshift;
        const int npg = pc.k1 > pc.k0 ? ((pc.k1 - 1) >> pshift) - pg0 + 1 : 0;
#pragma unroll
        for (int i = 0; i < PTR; ++i) {
            const int idx = lane + 64 * i;
            pr[i] = idx < npg ? P.page_table[pc.pt_base + pg0 + idx] : 0;
        }
    };
    auto store_pages = [&](int buf, const int32_t (&pr)[PTR]) {
#pragma unroll
        for (int i = 0; i < PTR; ++i) sPT[buf][lane + 64 * i] = pr[i];
    };

    // query operands of a piece (zeros for rows beyond its draft rows)
    vec8 qf[NT][KCALLS];
    auto load_q = [&](const Piece& pc) {
        const int kvh = pc.head_flags & kPieceHeadMask;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int nn = nt * 16 + m16;
            const int tl = nn / G, hg = nn - tl * G;
            const bool valid = tl < pc.n_q;
            const uint16_t* qp = P.q + ((int64_t)(pc.q_row0 + (valid ? tl : 0)) * P.n_q_heads + kvh * G + hg) * D + g * 8;
#pragma unroll
            for (int c = 0; c < KCALLS; ++c) {
                u32x4 v = valid ? *(const u32x4*)(qp + c * 32) : u32x4{0, 0, 0, 0};
                qf[nt][c] = __builtin_bit_cast(vec8, v);
            }
        }
    };

    // K/V rows of 32 keys starting at kb of the piece described by (buf, pg0, k1, head_off)
    u32x4 Kr[KLOADS], Vr[8];
    auto row_ptr = [&](const uint16_t* pool, int buf, int pg0, int k1, int64_t head_off, int key) -> const uint16_t* {
        key = min(key, k1 - 1);   // keys past the piece's end are masked; fetch a valid row instead
        const int pg = sPT[buf][(key >> pshift) - pg0];
        return pool + (int64_t)pg * P.page_stride + head_off + (int64_t)(key & pmask) * P.token_stride;
    };
    // With pages of 16 tokens or more, a full 32-key block that starts on a multiple of 32 is two runs
    // of 16 rows at the token pitch (two pages, or two halves of one): two wavefront-uniform base
    // addresses plus per-lane offsets that never change, no per-lane address arithmetic.  Anything
    // else takes the general path.
    const bool tile_layout = pshift >= 4;
    const uint32_t ts2 = (uint32_t)P.token_stride * 2;                                  // token pitch in bytes
    const uint32_t k_lane_off = (uint32_t)(lane / DCH) * ts2 + (uint32_t)(lane % DCH) * 16;   // K: a load covers 64/DCH rows
    const uint32_t v_lane_off = (uint32_t)(g * 4) * ts2 + (uint32_t)(m16 % DCH) * 16;         // V: a lane's column chunk, keys 4g..
    auto page_bases = [&](const uint16_t* pool, int buf, int pg0, int64_t head_off, int kb, const char*& a, const char*& b) {
        const int pga = __builtin_amdgcn_readfirstlane(sPT[buf][(kb >> pshift) - pg0]);
        const int pgb = __builtin_amdgcn_readfirstlane(sPT[buf][((kb + 16) >> pshift) - pg0]);
        a = (const char*)(pool + (int64_t)pga * P.page_stride + head_off + (int64_t)(kb & pmask) * P.token_stride);
        b = (const char*)(pool + (int64_t)pgb * P.page_stride + head_off + (int64_t)((kb + 16) & pmask) * P.token_stride);
    };
    auto load_k_runs = [&](const char* a, const char* b) {   // K of a block given as two runs of 16 rows
        constexpr int KPI = 64 / DCH;            // keys per load instruction
#pragma unroll
        for (int i = 0; i < KLOADS; ++i) {
            const int key = i * KPI;             // first key of this instruction within the block
            Kr[i] = stream_load((key < 16 ? a : b) + (int64_t)(key & 15) * ts2, k_lane_off);
        }
    };
    auto load_v_runs = [&](const char* a, const char* b) {
#pragma unroll
        for (int j = 0; j < 8; ++j) Vr[j] = stream_load((j < 4 ? a : b) + (int64_t)(j & 3) * ts2, v_lane_off);
    };
    auto load_k = [&](int buf, int pg0, int k1, int64_t head_off, int kb) {
        if (tile_layout && !(kb & 31) && kb + 32 <= k1) {
            const char *a, *b;
            page_bases(P.k_pool, buf, pg0, head_off, kb, a, b);
            load_k_runs(a, b);
        } else {
#pragma unroll
            for (int i = 0; i < KLOADS; ++i) {
                const int f = i * 64 + lane;
                Kr[i] = stream_load(row_ptr(P.k_pool, buf, pg0, k1, head_off, kb + f / DCH) + (f % DCH) * 8);
            }
        }
    };
    auto load_v = [&](int buf, int pg0, int k1, int64_t head_off, int kb) {
        if (tile_layout && !(kb & 31) && kb + 32 <= k1) {
            const char *a, *b;
            page_bases(P.v_pool, buf, pg0, head_off, kb, a, b);
            load_v_runs(a, b);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int kl = (j >> 2) * 16 + g * 4 + (j & 3);
                Vr[j] = stream_load(row_ptr(P.v_pool, buf, pg0, k1, head_off, kb + kl) + (m16 % DCH) * 8);
            }
        }
    };

    // ---- start-up.  The share's first K/V block is requested at once when the host has resolved it (its page ids
    // come with the share): the descriptors, page ids and queries that the rest needs take three dependent round
    // trips, and the block arrives while they are made.
    typedef const int32_t __attribute__((address_space(4)))* ConstInts;
    const ConstInts first = (ConstInts)(uintptr_t)(P.share_first + (int64_t)share * 4);
    const int first_pga = first[0], first_pgb = first[1], first_kvh = first[2], first_k0 = first[3];
    const bool ahead = first_k0 >= 0;
    if (ahead) {
        const int64_t head_off = (int64_t)first_kvh * P.head_stride;
        const int64_t oa = (int64_t)first_pga * P.page_stride + head_off + (int64_t)(first_k0 & pmask) * P.token_stride;
        const int64_t ob = (int64_t)first_pgb * P.page_stride + head_off + (int64_t)((first_k0 + 16) & pmask) * P.token_stride;
        load_k_runs((const char*)(P.k_pool + oa), (const char*)(P.k_pool + ob));
        load_v_runs((const char*)(P.v_pool + oa), (const char*)(P.v_pool + ob));
    }
    // The first four descriptors, page ids of the first three pieces in LDS
    Piece cp, p1, p2, p3;
    fetch_piece(0, cp);
    fetch_piece(1, p1);
    fetch_piece(2, p2);
    fetch_piece(3, p3);
    int next_piece = 4;
    int32_t pr[PTR];
    load_pages(cp, pr);
    store_pages(0, pr);
    load_pages(p1, pr);
    store_pages(1, pr);
    load_pages(p2, pr);
    store_pages(2, pr);
    bool pr_pending = false;   // pr holds page ids that still have to go to LDS
    load_q(cp);
    __syncthreads();

    f32x4 O[NT][8];
    float m_run[NT], l_run[NT];
    int lim[NT];
    uint64_t anc[NT];   // TREE: draft keys (bit u = key prefix + u) each row may see
    int pfx = 0;        // TREE: the request's prefix length
    int cb = 0;   // LDS page-id buffer of the current piece; the next piece's is (cb + 1) % 3
    if (!ahead) {
        const int64_t head = (int64_t)(cp.head_flags & kPieceHeadMask) * P.head_stride;
        load_k(cb, cp.k0 >> pshift, cp.k1, head, cp.k0);
        load_v(cb, cp.k0 >> pshift, cp.k1, head, cp.k0);
    }

    while (true) {
        // ---- per piece: visibility limits; fresh accumulators unless it continues the previous piece
        const bool carry_in = cp.head_flags & kPieceCarryIn;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int tl = (nt * 16 + m16) / G;
            lim[nt] = tl < cp.n_q ? min(cp.k1, cp.causal0 + tl) : cp.k0;
            if (TREE) {
                const u32x4 rec = *(const u32x4*)(P.tree_rows + (int64_t)(cp.q_row0 + (tl < cp.n_q ? tl : 0)) * 4);
                anc[nt] = (uint64_t)rec[0] | ((uint64_t)rec[1] << 32);
                pfx = __builtin_amdgcn_readfirstlane((int)rec[2]);
            }
            if (!carry_in) {
                m_run[nt] = kNegBig;
                l_run[nt] = 0.f;
#pragma unroll
                for (int jd = 0; jd < 8; ++jd) O[nt][jd] = f32x4{0, 0, 0, 0};
            }
        }
        // keys below this are visible to every row
        const int full_end = TREE ? min(min(cp.k1, cp.causal0), pfx) : min(cp.k1, cp.causal0);
        const bool more = p1.k1 > p1.k0;               // another piece follows this one
        const bool new_q = more && !(p1.head_flags & kPieceCarryIn);

        for (int kb = cp.k0; kb < cp.k1; kb += 32) {
            // The block after this one: the next 32 keys of this piece, or the first of the next
            // piece.  With nothing left the current block is fetched once more (valid memory, unused).
            const bool last = kb + 32 >= cp.k1;
            const bool hop = last && more;
            const int s_buf = hop ? (cb == 2 ? 0 : cb + 1) : cb;
            const int s_pg0 = hop ? (p1.k0 >> pshift) : (cp.k0 >> pshift);
            const int s_k1 = hop ? p1.k1 : cp.k1;
            const int64_t s_head = (int64_t)((hop ? p1.head_flags : cp.head_flags) & kPieceHeadMask) * P.head_stride;
            const int s_kb = hop ? p1.k0 : (last ? kb : kb + 32);

            // ---- K: registers -> LDS in operand shape
            __syncthreads();
#pragma unroll
            for (int i = 0; i < KLOADS; ++i) {
                const int f = i * 64 + lane;
                *(u32x4*)&sK[(f / DCH) * LROW + (f % DCH) * 8] = Kr[i];
            }
            // Page ids asked for during the previous piece's last block are older than the K rows just
            // consumed, so they have arrived: they belong to the piece two after this one and take the
            // LDS buffer of the piece before this one.
            if (pr_pending) {
                store_pages(cb == 0 ? 2 : cb - 1, pr);
                pr_pending = false;
            }
            __syncthreads();
            // During the last block, ask for the page ids of the piece three after this one (its
            // descriptor was fetched when this piece began).  Issued before the K/V rows below so that
            // waiting for those rows also covers these.
            if (last && (p3.k1 > p3.k0)) {
                load_pages(p3, pr);
                pr_pending = true;
            }
            load_k(s_buf, s_pg0, s_k1, s_head, s_kb);

            // ---- S^T = K Q^T
            f32x4 S[2][NT];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) S[t][nt] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int c = 0; c < KCALLS; ++c)      // the two tiles alternate, so consecutive MFMAs are independent
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const vec8 a = __builtin_bit_cast(vec8, *(const u32x4*)&sK[(t * 16 + m16) * LROW + (c * 4 + g) * 8]);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        S[t][nt] = E::mfma(a, qf[nt][c], S[t][nt]);
                }
            // the queries are no longer needed after the last block: fetch the next piece's if they differ
            if (last && new_q) load_q(p1);

            // ---- online softmax; lane (row, g) holds keys kb + t*16 + g*4 + r
            const bool full = kb + 32 <= full_end;
            vec8 Pb[NT];
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
                        if (TREE && key >= pfx && !((anc[nt] >> ((key - pfx) & 63)) & 1)) s[e] = -INFINITY;
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
                u32x4 pk = {E::pack(p[0], p[1]), E::pack(p[2], p[3]), E::pack(p[4], p[5]), E::pack(p[6], p[7])};
                Pb[nt] = __builtin_bit_cast(vec8, pk);
            }

            // ---- V: 8x8 transpose of 16-bit values inside each lane, then O^T += V^T P^T
            // (in two halves of four head dims, to keep the transposed copy small)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                u32x4 Vt[4];
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const int jd = hh * 4 + j4;
                    const uint32_t sel = (jd & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
                    for (int kp = 0; kp < 4; ++kp)
                        Vt[j4][kp] = __builtin_amdgcn_perm(Vr[2 * kp + 1][jd >> 1], Vr[2 * kp][jd >> 1], sel);
                }
                if (hh == 1) load_v(s_buf, s_pg0, s_k1, s_head, s_kb);
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const vec8 a = __builtin_bit_cast(vec8, Vt[j4]);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        O[nt][hh * 4 + j4] = E::mfma(a, Pb[nt], O[nt][hh * 4 + j4]);
                }
            }
        }

        // ---- result of this piece, unless the next piece carries on with the same accumulators:
        // parked in LDS.  Lane (row, g) holds, per jd, head dims (g*4 + r)*8 + jd, r = 0..3.
        if (!(cp.head_flags & kPieceCarryOut)) {
            const bool direct = cp.head_flags & kPieceDirect;
            const int need = NT * (direct ? 1 : 2);
            if (st_units + need > kStageUnits || st_n == kStageEntries) flush();
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float l = l_run[nt];
                l += __shfl_xor(l, 16);
                l += __shfl_xor(l, 32);
                u32x4* dst = sStage + (st_units + nt * (direct ? 1 : 2)) * 256 + lane;
                if (direct) {
                    const float inv = 1.0f / l;
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        dst[r * 64] = u32x4{E::pack(O[nt][0][r] * inv, O[nt][1][r] * inv), E::pack(O[nt][2][r] * inv, O[nt][3][r] * inv),
                                            E::pack(O[nt][4][r] * inv, O[nt][5][r] * inv), E::pack(O[nt][6][r] * inv, O[nt][7][r] * inv)};
                } else {
#pragma unroll
                    for (int jd = 0; jd < 8; ++jd) dst[jd * 64] = __builtin_bit_cast(u32x4, O[nt][jd]);
                    if (g == 0) {
                        sStageML[st_n][(nt * 16 + m16) * 2] = m_run[nt];
                        sStageML[st_n][(nt * 16 + m16) * 2 + 1] = l;
                    }
                }
            }
            if (lane == 0) {
                sStageDesc[st_n][0] = cp.head_flags;
                sStageDesc[st_n][1] = cp.q_row0;
                sStageDesc[st_n][2] = cp.n_q;
                sStageDesc[st_n][3] = cp.out_base;
            }
            ++st_n;
            st_units += need;
        }
        if (!more) break;

        // ---- move on to the next piece; fetch one more descriptor
        cb = cb == 2 ? 0 : cb + 1;
        cp = p1;
        p1 = p2;
        p2 = p3;
        fetch_piece(next_piece++, p3);
    }
    flush();
    }
    if (P.n_queued == 0) break;
    int next = 0;
    if (lane == 0) next = atomicAdd(P.queue, 1);
    next = __builtin_amdgcn_readfirstlane(next);
    if (next >= P.n_queued) break;
    share = gridDim.x + next;
    __syncthreads();
    }
}

template <int D, int NT, bool TREE, class E>
__global__ __launch_bounds__(64) void verify_attn_kernel(AttnParams P) {
    verify_attn_body<D, NT, TREE, E>(P);
}
// the same with the tables of the call in the kernel arguments (small calls)
template <int D, int NT, bool TREE, class E>
__global__ __launch_bounds__(64) void verify_attn_small_kernel(AttnParams P, InlineTables) {
    use_inline_tables<TREE>(P);
    verify_attn_body<D, NT, TREE, E>(P);
}

// Grouped-query variant: with G query heads per KV head a strip has up to 64 (draft row x query
// head) rows, four MFMA column tiles, whose arithmetic per key a single wavefront cannot hide behind
// its own loads.  A workgroup of eight wavefronts (one per CU, two per SIMD) therefore splits the
// work by kind:
//   * wavefronts 4..7 stream: each owns 32 keys of every 128-key block, keeps the loads of two
//     blocks in flight in two register sets (K and V both as 1 KiB-contiguous loads), and parks the
//     older set in LDS -- K in MFMA operand shape, V already transposed into MFMA operands (the 8x8
//     register transpose of the single-wavefront kernel, done once here for all readers) -- into
//     one of two stages, alternating;
//   * wavefronts 0..3 compute: wavefront t owns row tile t (16 rows) of the strip and works through
//     the four 32-key sub-blocks of the stage the streamers have just filled.
// One barrier per block hands a stage over (block i is parked before that barrier and consumed after
// it, while block i+1 is parked into the other stage), so the streamers run one block ahead in LDS and
// two more in registers, their load stream never waits for arithmetic, and the stores and query
// loads of the computing wavefronts never sit between a streamer's load and its wait.  Both kinds
// walk the same list of pieces of the workgroup's share; every K/V byte is fetched from HBM once.
constexpr int kGroupWaves = 8;
// Result rows are written once and never read by this kernel.  They leave as whole rows per store instruction
// and as write-through stores: lines that wait in the cache to be written back -- and rows written in pieces by
// several instructions -- cost a saturated read stream several times what whole lines written through at once do
// (measured: 18.9 MB of rows during a 4 GiB stream cost 92 us as plain stores, 22 us written through).
// (The two idle cycles behind the store: a vector instruction must not overwrite the data registers of a store
// of more than 8 bytes in the two cycles after it, and the compiler, which leaves such gaps behind its own
// stores, does not look inside an asm statement.)
__device__ __forceinline__ void store_row_piece(void* p, u32x4 w) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(w) : "memory");
}

template <int D, bool TREE, class E>
__device__ __forceinline__ void verify_attn_group_body(const AttnParams& P) {
    typedef typename E::vec8 vec8;
    constexpr int DCH = D / 8;
    constexpr int KCALLS = D / 32;
    constexpr int KLOADS = DCH / 2;
    constexpr int LROW = D + 8;
    constexpr int BK = 128;          // keys per block: 32 per streaming wavefront
    static_assert(BK == block_keys(2), "the planner balances shares in blocks of this kernel's size");
    constexpr int PTR = (kMaxPiecePages + 63) / 64;
    __shared__ __attribute__((aligned(16))) uint16_t sK[2][4][32 * LROW];
    __shared__ u32x4 sVt[2][4][8][64];   // V of each sub-block as MFMA operands: [head dim within chunk][lane]
    __shared__ int32_t sPT[3][PTR * 64];
    __shared__ u32x4 sOut[4][16 * 17];   // per computing wavefront: its 16 result rows (16 pieces of 16 bytes + 1 of padding each)

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m16 = lane & 15, g = lane >> 4;
    const int G = P.group;
    const int pshift = P.page_shift;
    const int pmask = (1 << pshift) - 1;

    // One share per workgroup: the planner queues no chunks for this kernel (its cuts cost more in partial
    // results than the evening-out of the ends saves).
    const int share = blockIdx.x;
    const int pc_begin = P.wave_begin[share], pc_end = P.wave_begin[share + 1];
    if (pc_begin >= pc_end) return;   // (the same for the whole workgroup; shares are never empty)
    auto fetch_piece = [&](int r, Piece& pc) {
        if (pc_begin + r < pc_end) {
            typedef const int32_t __attribute__((address_space(4)))* ConstWords;
            const ConstWords w = (ConstWords)(uintptr_t)(P.pieces + pc_begin + r);
            pc = Piece{w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]};
        } else {
            pc = Piece{0, 0, 0, 0, 0, 0, 0, 0};
        }
    };
    // Both kinds of wavefront pass the same barriers: three while the streamers start up and one per block.

    if (wave >= 4) {
        // ================================================================== streaming wavefronts
        __builtin_amdgcn_s_setprio(2);   // few instructions, all of them on the critical path of the memory stream
        const int w = wave - 4;          // this wavefront's 32 keys of every block
        // page ids are fetched by the first streaming wavefront for all four
        auto load_pages = [&](const Piece& pc, int32_t (&pr)[PTR]) {
            const int pg0 = pc.k0 >> pshift;
            const int npg = pc.k1 > pc.k0 ? ((pc.k1 - 1) >> pshift) - pg0 + 1 : 0;
#pragma unroll
            for (int i = 0; i < PTR; ++i) {
                const int idx = lane + 64 * i;
                pr[i] = (w == 0 && idx < npg) ? P.page_table[pc.pt_base + pg0 + idx] : 0;
            }
        };
        auto store_pages = [&](int buf, const int32_t (&pr)[PTR]) {
            if (w == 0) {
#pragma unroll
                for (int i = 0; i < PTR; ++i) sPT[buf][lane + 64 * i] = pr[i];
            }
        };
        auto row_ptr = [&](const uint16_t* pool, int buf, int pg0, int k1, int64_t head_off, int key) -> const uint16_t* {
            key = min(key, k1 - 1);   // past the end: a valid row, masked later
            const int pg = sPT[buf][(key >> pshift) - pg0];
            return pool + (int64_t)pg * P.page_stride + head_off + (int64_t)(key & pmask) * P.token_stride;
        };
        const bool tile_layout = pshift >= 4;   // see the single-wavefront kernel
        const uint32_t ts2 = (uint32_t)P.token_stride * 2;
        const uint32_t k_lane_off = (uint32_t)(lane / DCH) * ts2 + (uint32_t)(lane % DCH) * 16;
        const uint32_t v_lane_off = (uint32_t)(g * 4) * ts2 + (uint32_t)(m16 % DCH) * 16;
        // One register set: this wavefront's 32 keys (kb + 32*w ...) of a block, K as 1 KiB-contiguous
        // loads, V as the same 16-byte column chunk of eight keys per lane (see the kernel above).
        struct RegSet {
            u32x4 Kr[KLOADS], Vr[8];
        };
        // this wavefront's 32 keys kw.. of a block as two runs of 16 rows in pages pga, pgb
        auto load_kv_runs = [&](RegSet& R, int pga, int pgb, int64_t head_off, int kw) {
            {
                const int64_t oa = (int64_t)pga * P.page_stride + head_off + (int64_t)(kw & pmask) * P.token_stride;
                const int64_t ob = (int64_t)pgb * P.page_stride + head_off + (int64_t)((kw + 16) & pmask) * P.token_stride;
                const char *ka = (const char*)(P.k_pool + oa), *kb_ = (const char*)(P.k_pool + ob);
                const char *va = (const char*)(P.v_pool + oa), *vb = (const char*)(P.v_pool + ob);
                constexpr int KPI = 64 / DCH;
#pragma unroll
                for (int i = 0; i < KLOADS; ++i) {
                    const int key = i * KPI;
                    R.Kr[i] = stream_load((key < 16 ? ka : kb_) + (int64_t)(key & 15) * ts2, k_lane_off);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) R.Vr[j] = stream_load((j < 4 ? va : vb) + (int64_t)(j & 3) * ts2, v_lane_off);
            }
        };
        auto load_kv = [&](RegSet& R, int buf, int pg0, int k1, int64_t head_off, int kb) {
            const int kw = kb + 32 * w;
            if (tile_layout && !(kb & 31) && kb + BK <= k1) {
                const int pga = __builtin_amdgcn_readfirstlane(sPT[buf][(kw >> pshift) - pg0]);
                const int pgb = __builtin_amdgcn_readfirstlane(sPT[buf][((kw + 16) >> pshift) - pg0]);
                load_kv_runs(R, pga, pgb, head_off, kw);
            } else {
#pragma unroll
                for (int i = 0; i < KLOADS; ++i) {
                    const int f = i * 64 + lane;
                    R.Kr[i] = stream_load(row_ptr(P.k_pool, buf, pg0, k1, head_off, kw + f / DCH) + (f % DCH) * 8);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int kl = (j >> 2) * 16 + g * 4 + (j & 3);
                    R.Vr[j] = stream_load(row_ptr(P.v_pool, buf, pg0, k1, head_off, kw + kl) + (m16 % DCH) * 8);
                }
            }
        };
        auto park = [&](const RegSet& R, int stage) {
#pragma unroll
            for (int i = 0; i < KLOADS; ++i) {
                const int f = i * 64 + lane;
                *(u32x4*)&sK[stage][w][(f / DCH) * LROW + (f % DCH) * 8] = R.Kr[i];
            }
            // V: 8x8 transpose of 16-bit values inside each lane, done once here for all readers
#pragma unroll
            for (int jd = 0; jd < 8; ++jd) {
                const uint32_t sel = (jd & 1) ? 0x07060302u : 0x05040100u;
                u32x4 vt;
#pragma unroll
                for (int kp = 0; kp < 4; ++kp) vt[kp] = __builtin_amdgcn_perm(R.Vr[2 * kp + 1][jd >> 1], R.Vr[2 * kp][jd >> 1], sel);
                sVt[stage][w][jd][lane] = vt;
            }
        };

        // The load cursor: the piece it is in (c0), the three after it, the page-id buffer of c0 and the
        // next block's first key.  Page ids of the piece three ahead are requested while the last block
        // of c0 is issued (ahead of that block's K/V loads, so that the K/V loads stay the youngest) and
        // stored one step later into the buffer c0 has just left.
        // The share's first block is requested at once when the host has resolved it (its page ids come with the
        // share), as in the single-wavefront kernel: it arrives while the descriptors and page ids are fetched.
        RegSet A, B;
        typedef const int32_t __attribute__((address_space(4)))* ConstInts;
        const ConstInts first = (ConstInts)(uintptr_t)(P.share_first + (int64_t)share * 10);
        const int wu = __builtin_amdgcn_readfirstlane(w);
        const int first_pga = first[2 * wu], first_pgb = first[2 * wu + 1], first_kvh = first[8], first_k0 = first[9];
        bool ahead = first_k0 >= 0;
        if (ahead) load_kv_runs(A, first_pga, first_pgb, (int64_t)first_kvh * P.head_stride, first_k0 + 32 * w);
        Piece c0, c1, c2, c3;
        fetch_piece(0, c0);
        fetch_piece(1, c1);
        fetch_piece(2, c2);
        fetch_piece(3, c3);
        int next_piece = 4;
        int32_t pr[PTR];
        load_pages(c0, pr);
        store_pages(0, pr);
        load_pages(c1, pr);
        store_pages(1, pr);
        load_pages(c2, pr);
        store_pages(2, pr);
        bool pr_pending = false;
        int cb = 0, kb = c0.k0;
        __syncthreads();                 // barrier 0: the page ids are in place
        auto issue = [&](RegSet& R) {
            const bool last = kb + BK >= c0.k1;
            if (pr_pending) {
                store_pages(cb == 0 ? 2 : cb - 1, pr);
                pr_pending = false;
            }
            if (last && c3.k1 > c3.k0) {
                load_pages(c3, pr);
                pr_pending = true;
            }
            if (!ahead) load_kv(R, cb, c0.k0 >> pshift, c0.k1, (int64_t)(c0.head_flags & kPieceHeadMask) * P.head_stride, kb);
            ahead = false;
            if (!last) {
                kb += BK;
            } else if (c1.k1 > c1.k0) {
                cb = cb == 2 ? 0 : cb + 1;
                c0 = c1;
                c1 = c2;
                c2 = c3;
                fetch_piece(next_piece++, c3);
                kb = c0.k0;
            }   // else: the share is exhausted; the cursor stays, later loads repeat its last block and are never parked
        };
        // (a barrier after each of the first two issues as well: a page-id buffer is rewritten one step
        // after the cursor has left it, and every step must be over in all four wavefronts by then)
        issue(A);
        __syncthreads();                 // barrier 1
        issue(B);
        __syncthreads();                 // barrier 2
        int n_blocks = 0;                // blocks of the whole share
        for (int r = 0; pc_begin + r < pc_end; ++r) {
            Piece t;
            fetch_piece(r, t);
            n_blocks += (t.k1 - t.k0 + BK - 1) / BK;
        }
        for (int i = 0; i < n_blocks; i += 2) {
            park(A, 0);
            issue(A);
            __syncthreads();             // barrier i + 3: block i is in stage 0
            if (i + 1 < n_blocks) {
                park(B, 1);
                issue(B);
                __syncthreads();         // barrier i + 4: block i + 1 is in stage 1
            }
        }
        return;
    }

    // ====================================================================== computing wavefronts
    const int tile = wave;               // the row tile (16 rows of the strip) this wavefront owns
    vec8 qf[KCALLS];
    uint64_t anc_n = 0;                  // TREE: the next piece's ancestor mask and prefix length
    int pfx_n = 0;
    auto load_q = [&](const Piece& pc, vec8 (&q)[KCALLS]) {
        const int kvh = pc.head_flags & kPieceHeadMask;
        const int nn = tile * 16 + m16;
        const int tl = nn / G, hg = nn - tl * G;
        const bool valid = tl < pc.n_q;
        const uint16_t* qp = P.q + ((int64_t)(pc.q_row0 + (valid ? tl : 0)) * P.n_q_heads + kvh * G + hg) * D + g * 8;
#pragma unroll
        for (int c = 0; c < KCALLS; ++c) {
            u32x4 v = valid ? *(const u32x4*)(qp + c * 32) : u32x4{0, 0, 0, 0};
            q[c] = __builtin_bit_cast(vec8, v);
        }
        if (TREE) {
            const u32x4 rec = *(const u32x4*)(P.tree_rows + (int64_t)(pc.q_row0 + (valid ? tl : 0)) * 4);
            anc_n = (uint64_t)rec[0] | ((uint64_t)rec[1] << 32);
            pfx_n = (int)rec[2];
        }
    };
    Piece cp, p1;
    fetch_piece(0, cp);
    fetch_piece(1, p1);
    int next_piece = 2;
    load_q(cp, qf);
    // (reading the query registers here puts the wait for them in front of the loop: inside it no wait for a
    // memory operation may follow a store, see below)
#pragma unroll
    for (int c = 0; c < KCALLS; ++c) asm volatile("" : "+v"(qf[c]));
    uint64_t anc = anc_n;                // TREE: draft keys (bit u = key prefix + u) this lane's row may see
    int pfx = __builtin_amdgcn_readfirstlane(pfx_n);
    f32x4 O[8];
    float m_run = kNegBig, l_run = 0.f;
    int blk = 0;                          // blocks of the share so far: block i sits in stage i & 1
    __syncthreads();                      // barriers 0, 1, 2: the streamers' start-up
    __syncthreads();
    __syncthreads();

    while (true) {
        const bool active = tile * 16 < cp.n_q * G;     // narrower strips leave the upper tiles idle
        const int nn = tile * 16 + m16;                  // this lane's row of the strip's (draft row x head) rows
        const int tl = nn / G;
        const int lim = tl < cp.n_q ? min(cp.k1, cp.causal0 + tl) : cp.k0;
        if (!(cp.head_flags & kPieceCarryIn)) {
            m_run = kNegBig;
            l_run = 0.f;
#pragma unroll
            for (int jd = 0; jd < 8; ++jd) O[jd] = f32x4{0, 0, 0, 0};
        }
        const int full_end = TREE ? min(min(cp.k1, cp.causal0), pfx) : min(cp.k1, cp.causal0);
        const bool more = p1.k1 > p1.k0;

        auto block = [&](int kb, int st, bool last) {
            // The block as a whole -- scores of all four sub-blocks, one test of the exponent reference, all
            // exponentials, all of P.V -- in straight-line code, so that the LDS reads, matrix and vector
            // instructions of different sub-blocks overlap (this wavefront has its SIMD almost to itself
            // and nothing else would hide their latencies).  Rows of the block beyond the piece's end are
            // copies of its last key (see the streamers) and fall to the mask like every key beyond `lim`.
            f32x4 S[4][2];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                S[sb][0] = f32x4{0, 0, 0, 0};
                S[sb][1] = f32x4{0, 0, 0, 0};
#pragma unroll
                for (int c = 0; c < KCALLS; ++c)
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const vec8 a = __builtin_bit_cast(vec8, *(const u32x4*)&sK[st][sb][(t * 16 + m16) * LROW + (c * 4 + g) * 8]);
                        S[sb][t] = E::mfma(a, qf[c], S[sb][t]);
                    }
            }
            // The queries are no longer needed after the piece's last block: the next piece's are requested
            // here, straight into the same registers, so that they arrive behind the rest of this block.
            if (last) load_q(p1, qf);
            float sc[4][8];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                for (int e = 0; e < 8; ++e) sc[sb][e] = S[sb][e >> 2][e & 3];
            if (kb + BK > full_end) {
#pragma unroll
                for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int key = kb + 32 * sb + (e >> 2) * 16 + g * 4 + (e & 3);
                        if (key >= lim) sc[sb][e] = -INFINITY;
                        if (TREE && key >= pfx && !((anc >> ((key - pfx) & 63)) & 1)) sc[sb][e] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                for (int e = 0; e < 8; ++e) mx = fmaxf(mx, sc[sb][e]);
            // The exponent reference m_run (one value per row, the same in the row's four lanes) follows
            // the running maximum lazily: it moves (and the accumulators are rescaled) only when some
            // score has grown past it by more than kSlack, so exp2(score - m_run) stays below 2^kSlack and
            // most blocks skip the rescale -- and with it the two cross-lane exchanges that make a row's
            // maximum out of its lanes' maxima.
            if (__any(mx * P.scale_log2 > m_run + kSlack)) {
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run, mx * P.scale_log2);
                const float alpha = fast_exp2(m_run - m_new);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int jd = 0; jd < 8; ++jd) O[jd] *= alpha;
            }
            vec8 Pb[4];
            float sum = 0.f;
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                float p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = fast_exp2(sc[sb][e] * P.scale_log2 - m_run);
                    sum += p[e];
                }
                const u32x4 pk = {E::pack(p[0], p[1]), E::pack(p[2], p[3]), E::pack(p[4], p[5]), E::pack(p[6], p[7])};
                Pb[sb] = __builtin_bit_cast(vec8, pk);
            }
            l_run += sum;
#pragma unroll
            for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                for (int jd = 0; jd < 8; ++jd)
                    O[jd] = E::mfma(__builtin_bit_cast(vec8, sVt[st][sb][jd][lane]), Pb[sb], O[jd]);
        };
        // All blocks but the last in a loop that holds no memory load, then the last one, which requests the
        // next piece's queries: kept apart so that the wait for those queries is not carried into the loop
        // (where, placed in front of the first use of the queries, it would follow the stores below).
        int kb = cp.k0;
        for (; kb + BK < cp.k1; kb += BK) {
            __syncthreads();              // barrier blk + 3: the streamers have parked this block
            if (active) block(kb, blk & 1, false);
            ++blk;
        }
        __syncthreads();
        if (active) block(kb, blk & 1, true);
        ++blk;

        // The next piece's queries must have ARRIVED before this piece's rows are stored: loads and stores
        // share one in-order counter, so any wait for a load that comes after the stores is a wait for the
        // stores -- several microseconds under a saturated read stream, more than the one block of slack this
        // wavefront has before the streamers stall at the next barrier.  The empty statement below reads the
        // query registers, which puts the wait for them here; after the stores this wavefront waits for no
        // memory operation until the end of the next piece.
        if (!active) load_q(p1, qf);
#pragma unroll
        for (int c = 0; c < KCALLS; ++c) asm volatile("" : "+v"(qf[c]));
        anc = anc_n;
        pfx = __builtin_amdgcn_readfirstlane(pfx_n);
        if (!(cp.head_flags & kPieceCarryOut) && active) {
            const int kvh = cp.head_flags & kPieceHeadMask;
            float l = l_run;
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            // Rows leave through a wavefront-private LDS tile, so that every store instruction writes whole rows
            // (lane (row, g) parks its four 16-byte pieces of row `row`; lane L of instruction k then takes piece
            // L % 16 of row 4 k + L / 16), written through (see store_row_piece).  A partial row is the row
            // normalised by its own sum, as half precision, next to its (maximum, sum) pair.
            const bool direct = cp.head_flags & kPieceDirect;
            const float inv = l > 0.f ? 1.0f / l : 0.f;          // (a partial row that saw no key: all zero, weight zero)
            u32x4* tilebuf = sOut[tile];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const u32x4 w = direct ? u32x4{E::pack(O[0][r] * inv, O[1][r] * inv), E::pack(O[2][r] * inv, O[3][r] * inv),
                                               E::pack(O[4][r] * inv, O[5][r] * inv), E::pack(O[6][r] * inv, O[7][r] * inv)}
                                       : u32x4{F16::pack(O[0][r] * inv, O[1][r] * inv), F16::pack(O[2][r] * inv, O[3][r] * inv),
                                               F16::pack(O[4][r] * inv, O[5][r] * inv), F16::pack(O[6][r] * inv, O[7][r] * inv)};
                tilebuf[m16 * 17 + g * 4 + r] = w;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int row = k * 4 + g, nr = tile * 16 + row;
                const int tr = nr / G, hr = nr - tr * G;
                const u32x4 w = tilebuf[row * 17 + m16];
                if (tr < cp.n_q && m16 < DCH) {
                    uint16_t* op = direct ? P.o + ((int64_t)(cp.q_row0 + tr) * P.n_q_heads + kvh * G + hr) * D + m16 * 8
                                          : P.part_o + ((int64_t)cp.out_base + nr) * kPartRow + m16 * 8;
                    store_row_piece(op, w);
                }
            }
            if (!direct && tl < cp.n_q && g == 0) {
                const int64_t slot = (int64_t)cp.out_base + nn;
                P.part_ml[slot * 2] = m_run;
                P.part_ml[slot * 2 + 1] = l;
            }
        }
        if (!more) break;
        cp = p1;
        fetch_piece(next_piece++, p1);
    }
}

template <int D, bool TREE, class E>
__global__ __launch_bounds__(64 * kGroupWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void verify_attn_group_kernel(AttnParams P) {
    verify_attn_group_body<D, TREE, E>(P);
}
template <int D, bool TREE, class E>
__global__ __launch_bounds__(64 * kGroupWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void verify_attn_group_small_kernel(AttnParams P, InlineTables) {
    use_inline_tables<TREE>(P);
    verify_attn_group_body<D, TREE, E>(P);
}

// Join the partial results of one (request, KV head): Eq. (13) -- one denominator over all tokens
// of the original request.  Piece s left (m_s, l_s, O_s): l_s = sum of exp2(score - m_s) over its keys and
// O_s its own normalised output (half precision):  O = sum_s w_s O_s / sum_s w_s,  w_s = 2^(m_s-M) l_s.
// One wavefront per (task, draft row, query head of the group); lane (chunk, jp) owns head dims
// chunk*8 + 2*jp and +1.  Rows whose pieces were all written directly have no partial result and are
// left alone.
constexpr int kJoinWaves = 4;

template <int D, class E>
__device__ __forceinline__ void join_partials_body(const JoinParams& P) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int req = P.tasks[2 * blockIdx.x], kvh = P.tasks[2 * blockIdx.x + 1];
    const int G = P.group;
    const int row0 = P.q_offset[req], n_rows = P.q_offset[req + 1] - row0;
    const int sb = P.strip_begin[req], se = P.strip_begin[req + 1];
    const int chunk = lane & 15, jp = lane >> 4;
    const int e0 = chunk * 8 + 2 * jp;
    const bool active = chunk * 8 < D;

    {
        const int pair = blockIdx.y * kJoinWaves + wave;
        if (pair >= n_rows * G) return;
        const int t = pair / G, hg = pair - t * G;
        const int r = row0 + t;
        float M = kNegBig, den = 0.f, n0 = 0.f, n1 = 0.f;
        bool any = false;
        for (int s = sb; s < se; ++s) {
            const int first = P.ppos[(s * P.n_kv_heads + kvh) * 2], cnt = P.ppos[(s * P.n_kv_heads + kvh) * 2 + 1];
            const int tl = r - P.pieces[first].q_row0;
            if (tl < 0 || tl >= P.pieces[first].n_q) continue;
#pragma unroll 2
            for (int k = first; k < first + cnt; ++k) {
                const Piece pc = P.pieces[k];
                if (pc.head_flags & (kPieceCarryOut | kPieceDirect)) continue;
                const int64_t slot = (int64_t)pc.out_base + tl * G + hg;
                const float m = P.part_ml[slot * 2], l = P.part_ml[slot * 2 + 1];
                const f16x2 o = __builtin_bit_cast(f16x2, *(const uint32_t*)(P.part_o + slot * kPartRow + e0));
                const float Mn = fmaxf(M, m);
                const float a = fast_exp2(M - Mn), b = fast_exp2(m - Mn) * l;
                den = den * a + b;
                n0 = n0 * a + (float)o[0] * b;
                n1 = n1 * a + (float)o[1] * b;
                M = Mn;
                any = true;
            }
        }
        if (any && active) {
            const float inv = 1.0f / den;
            const int h = kvh * G + hg;
            uint32_t* op = reinterpret_cast<uint32_t*>(P.o + ((int64_t)r * P.n_q_heads + h) * D + chunk * 8 + 2 * jp);
            *op = E::pack(n0 * inv, n1 * inv);
        }
    }
}

template <int D, class E>
__global__ __launch_bounds__(64 * kJoinWaves) void join_partials_kernel(JoinParams P) {
    join_partials_body<D, E>(P);
}
template <int D, class E>
__global__ __launch_bounds__(64 * kJoinWaves) void join_partials_small_kernel(JoinParams P, InlineTables) {
    const char* base = inline_tables_base<JoinParams>();
    rebase(P.pieces, base);
    rebase(P.ppos, base);
    rebase(P.strip_begin, base);
    rebase(P.q_offset, base);
    rebase(P.tasks, base);
    join_partials_body<D, E>(P);
}

// Scatter the draft tokens' K and V rows into their page slots: one workgroup per packed row, 16
// bytes per lane and step, over all KV heads of K and then of V.
__device__ __forceinline__ void append_kv_body(const AppendParams& P, int row, int64_t slot) {
    const int64_t page = slot >> P.page_shift, in_page = slot & ((1 << P.page_shift) - 1);
    const int per_head = P.head_dim >> 3, per_pool = P.n_kv_heads * per_head;
    const int64_t dst0 = page * P.page_stride + in_page * P.token_stride;
    const int64_t src0 = (int64_t)row * P.n_kv_heads * P.head_dim;
    for (int c = threadIdx.x; c < 2 * per_pool; c += 256) {
        const bool is_v = c >= per_pool;
        const int cc = is_v ? c - per_pool : c;
        const int head = cc / per_head, col = (cc - head * per_head) * 8;
        const uint16_t* src = (is_v ? P.v_new : P.k_new) + src0 + (int64_t)cc * 8;
        uint16_t* dst = (is_v ? P.v_pool : P.k_pool) + dst0 + head * P.head_stride + col;
        // (non-temporal: rows left behind as dirty cache lines are written back in the middle of the attention
        // kernel's stream, which costs it more than the whole scatter takes)
        __builtin_nontemporal_store(*(const u32x4*)src, (u32x4*)dst);
    }
}

__global__ __launch_bounds__(256) void append_kv_kernel(AppendParams P) {
    append_kv_body(P, blockIdx.x, P.dst_slot[blockIdx.x]);
}
// the same with the destination slots in the kernel arguments (batches of up to kInlineAppendRows draft rows)
struct InlineSlots {
    int32_t slot[kInlineAppendRows];
};
__global__ __launch_bounds__(256) void append_kv_small_kernel(AppendParams P, InlineSlots s, int row0) {
    append_kv_body(P, row0 + blockIdx.x, s.slot[blockIdx.x]);
}

hipError_t launch_append(const AppendParams& p, const int64_t* dst_slot_host, hipStream_t stream) {
    if (p.n_rows <= 0) return hipSuccess;
    if (dst_slot_host && p.n_rows <= kInlineAppendRows * kInlineAppendLaunches) {
        // (kernels launched back to back start without a gap; an event record between two kernels costs more
        // than a second launch)
        for (int row0 = 0; row0 < p.n_rows; row0 += kInlineAppendRows) {
            const int n = std::min(kInlineAppendRows, p.n_rows - row0);
            InlineSlots s;
            for (int i = 0; i < n; ++i) {
                if (dst_slot_host[row0 + i] < 0 || dst_slot_host[row0 + i] > INT32_MAX) return hipErrorInvalidValue;
                s.slot[i] = (int32_t)dst_slot_host[row0 + i];
            }
            hipLaunchKernelGGL(append_kv_small_kernel, dim3((unsigned)n), dim3(256), 0, stream, p, s, row0);
        }
    } else {
        if (!p.dst_slot) return hipErrorInvalidValue;
        hipLaunchKernelGGL(append_kv_kernel, dim3((unsigned)p.n_rows), dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

template <int D, bool TREE, class E>
static const void* attn_kernel_ptr(int cls, bool small = false) {
    if (small)
        return cls == 0 ? (const void*)verify_attn_small_kernel<D, 1, TREE, E>
             : cls == 1 ? (const void*)verify_attn_small_kernel<D, 2, TREE, E> : (const void*)verify_attn_group_small_kernel<D, TREE, E>;
    return cls == 0 ? (const void*)verify_attn_kernel<D, 1, TREE, E>
         : cls == 1 ? (const void*)verify_attn_kernel<D, 2, TREE, E> : (const void*)verify_attn_group_kernel<D, TREE, E>;
}

hipError_t attn_resident_waves(int head_dim, int cls, int* n_waves) {
    // (the tree-mask and fp16 variants differ by a few registers at most and are launched with the same counts)
    const void* fn = head_dim == 128 ? attn_kernel_ptr<128, false, Bf16>(cls) : attn_kernel_ptr<64, false, Bf16>(cls);
    int per_cu = 0, dev = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, cls == 2 ? 64 * kGroupWaves : 64, 0);
    if (e == hipSuccess) e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    // the single-wavefront kernel streams best with one wavefront per SIMD: more wavefronts mean more,
    // shorter shares (more cuts and partial results) and the stream is not latency-bound
    if (cls < 2 && per_cu > 4) per_cu = 4;
    *n_waves = per_cu * prop.multiProcessorCount;
    return hipSuccess;
}

template <int D, class E>
static hipError_t launch_attn_d(const AttnParams& base, const Piece* const pieces_dev[3],
                                const int32_t* const wave_begin_dev[3], const int32_t* const share_first_dev[3],
                                const int32_t n_waves[3],
                                const int32_t n_queued[3], int32_t* queues_dev, const JoinParams& jp,
                                const InlineTables* tables, hipStream_t stream, LaunchTiming* timing) {
    int first_cls = -1, last_cls = -1;   // (one class per call in practice; with several, the time spans them all)
    for (int cls = 0; cls < 3; ++cls)
        if (n_waves[cls] > 0) {
            if (first_cls < 0) first_cls = cls;
            last_cls = cls;
        }
    if (timing) timing->second = false;
    for (int cls = 0; cls < 3; ++cls) {
        if (n_waves[cls] <= 0) continue;
        AttnParams p = base;
        p.pieces = pieces_dev[cls];
        p.wave_begin = wave_begin_dev[cls];
        p.share_first = share_first_dev[cls];
        p.queue = queues_dev + cls;
        p.n_queued = n_queued[cls];
        if (cls == 2 && p.n_queued != 0) return hipErrorInvalidValue;   // the grouped-query kernel takes no queued chunks
        if (p.inline_tables && p.n_queued != 0) return hipErrorInvalidValue;   // the chunk queue needs device memory
        dim3 grid((unsigned)n_waves[cls]);
        void* args[] = {&p, (void*)tables};
        const bool small = p.inline_tables != 0;
        const void* fn = p.tree_rows ? attn_kernel_ptr<D, true, E>(cls, small) : attn_kernel_ptr<D, false, E>(cls, small);   // (an offset when inline, never zero)
        hipError_t e = hipExtLaunchKernel(fn, grid, dim3(cls == 2 ? 64 * kGroupWaves : 64), args, 0, stream,
                                          timing && cls == first_cls ? timing->ev[0] : nullptr,
                                          timing && cls == last_cls ? timing->ev[1] : nullptr, 0);
        if (e != hipSuccess) return e;
    }
    if (jp.n_tasks > 0) {
        const int pair_groups = (jp.max_pairs + kJoinWaves - 1) / kJoinWaves;
        const dim3 grid(jp.n_tasks, pair_groups), block(64 * kJoinWaves);
        hipEvent_t e0 = timing ? timing->ev[2] : nullptr, e1 = timing ? timing->ev[3] : nullptr;
        if (jp.inline_tables) hipExtLaunchKernelGGL((join_partials_small_kernel<D, E>), grid, block, 0, stream, e0, e1, 0, jp, *tables);
        else hipExtLaunchKernelGGL((join_partials_kernel<D, E>), grid, block, 0, stream, e0, e1, 0, jp);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (timing) timing->second = true;
    }
    return hipSuccess;
}

hipError_t launch_attn(int head_dim, bool f16, const AttnParams& base, const Piece* const pieces_dev[3],
                       const int32_t* const wave_begin_dev[3], const int32_t* const share_first_dev[3],
                       const int32_t n_waves[3], const int32_t n_queued[3],
                       int32_t* queues_dev, const JoinParams& jp, const void* inline_tables, size_t inline_bytes,
                       hipStream_t stream, LaunchTiming* timing) {
    InlineTables storage;
    const InlineTables* tables = nullptr;
    if (inline_tables) {
        if (inline_bytes > kInlineTableBytes || !base.inline_tables) return hipErrorInvalidValue;
        memcpy(storage.bytes, inline_tables, inline_bytes);
        tables = &storage;
    } else if (base.inline_tables || jp.inline_tables) {
        return hipErrorInvalidValue;
    }
    if (head_dim == 128)
        return f16 ? launch_attn_d<128, F16>(base, pieces_dev, wave_begin_dev, share_first_dev, n_waves, n_queued, queues_dev, jp, tables, stream, timing)
                   : launch_attn_d<128, Bf16>(base, pieces_dev, wave_begin_dev, share_first_dev, n_waves, n_queued, queues_dev, jp, tables, stream, timing);
    if (head_dim == 64)
        return f16 ? launch_attn_d<64, F16>(base, pieces_dev, wave_begin_dev, share_first_dev, n_waves, n_queued, queues_dev, jp, tables, stream, timing)
                   : launch_attn_d<64, Bf16>(base, pieces_dev, wave_begin_dev, share_first_dev, n_waves, n_queued, queues_dev, jp, tables, stream, timing);
    return hipErrorInvalidValue;
}

}  // namespace spin
