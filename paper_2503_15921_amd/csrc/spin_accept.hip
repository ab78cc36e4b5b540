// Acceptance kernels of the verification step (verification phase of Sec. II-A2; the rule is
// the speculative-sampling one of the works the paper cites in Sec. I) for gfx950.
//
// Two launches:
//   row_stats_kernel      one workgroup per logits row: maximum, arg-max (lowest id on ties) and
//                         sum of exp(x - max) in float64.  Bound by reading the logits once from
//                         HBM (the second sweep of a row comes out of L2).
//   accept_finish_kernel  one workgroup per request: the first-reject scan over its draft rows,
//                         then the next token -- arg-max (greedy), or an inverse-CDF search over
//                         the residual max(0, p - q) / the bonus row by a workgroup prefix scan.
// All probabilities are float64, so that the accepted lengths and token ids can be compared bit
// for bit with a float64 CPU evaluation of the same rule.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "spin_device.h"

namespace spin {

constexpr int kStatThreads = 256;
constexpr int kSweepLoads = 4;       // 16-byte loads a lane of the statistics sweep keeps in flight
constexpr int kTreeThreads = 1024;   // workgroup of the tree rejection kernel
constexpr int kMaxRuns = 1024;       // run sums of the inverse-CDF search kept in LDS

struct MaxArg {
    float v;
    int32_t i;
};

__device__ __forceinline__ MaxArg better(MaxArg a, MaxArg b) {
    // larger value wins; equal values -> lower index
    if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
    return a;
}

// exp(d) in float64 for the sums and masses, d in [-700, 700]: d = (256 e + j) ln2/256 + r with
// |r| <= ln2/512, so exp(d) = 2^e * 2^(j/256) * exp(r) with a 256-entry table (in LDS) and a cubic for
// exp(r) (remainder r^4/24 < 1.4e-13 relative, the rounded ln2/256 adds 2.4e-14: four orders below what
// the accept decisions need, and about half the float64 instructions of the general routine).  The integer
// 256 e + j is read off the low word of d * 256/ln2 + 1.5 * 2^52, and 2^e goes into the table value's
// exponent field by an integer add.
constexpr double kExpMagic = 6755399441055744.0;   // 1.5 * 2^52

__device__ __forceinline__ double exp_table64_in_range(double d, const double* tab) {
    const double t = fma(d, 369.3299304675746, kExpMagic);                  // 256 / ln 2
    const double kd = t - kExpMagic;
    const int k = __double2loint(t);
    const double r = fma(kd, -0.0027076061740622863, d);                     // ln2/256 rounded: off by 9.1e-20, |kd| < 3e5
    double p = fma(r, 1.0 / 6.0, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    const double T = tab[k & 255];
    return __hiloint2double(__double2hiint(T) + ((k & ~255) << 12), __double2loint(T)) * p;
}

// The same for any d below 700: minus infinity and everything below -700 give exp(-700) < 1e-304.
__device__ __forceinline__ double exp_table64(double d, const double* tab) { return exp_table64_in_range(fmax(d, -700.0), tab); }

// Row statistics travel between workgroups of one launch (the one that arrives last at a request's counter
// reads what the others wrote, on whatever part of the chip they ran): they are written and read as
// device-scope atomic accesses, which go past the caches that are private to a part of the chip, so that
// no cache has to be written back or invalidated as a whole.
__device__ __forceinline__ void put_stats(const AcceptParams& P, int row, float mx, double sum, int32_t arg) {
    __hip_atomic_store(P.row_max + row, mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(P.row_sum + row, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(P.row_arg + row, arg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS of the row statistics (one workgroup of kStatThreads per logits row).
struct StatShared {
    MaxArg ma[kStatThreads / 64];
    double sum[kStatThreads / 64];
    float ref[kStatThreads / 64];
    double tab[256];               // 2^(j/256) for exp_table64
};

// Statistics of one logits row by a workgroup of kStatThreads threads: maximum, arg-max (lowest id on
// ties; greedy mode) or maximum and sum of exp(x - max) in float64 (rejection mode).  Leaves sh.tab filled
// in rejection mode.
// STREAM: the logits are read with non-temporal loads (batches whose logits do not fit the last-level cache anyway).
template <bool STREAM = false>
__device__ __forceinline__ void row_stats_body(const AcceptParams& P, int row, StatShared& sh) {
    MaxArg* const s_ma = sh.ma;
    double* const s_sum = sh.sum;
    float* const s_ref = sh.ref;
    double* const s_tab = sh.tab;
    const int n_target = P.n_rows + P.n_req;
    const float* x = row < n_target ? P.target_logits + (int64_t)row * P.vocab
                                    : P.draft_logits + (int64_t)(row - n_target) * P.vocab;
    const int V = P.vocab;
    const int tid = threadIdx.x;
    const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
    const float4* x4 = reinterpret_cast<const float4*>(x);
    const int g_lo = 0, g_hi = V / 4, e_lo = 0, e_hi = V, out = row;

    if (P.mode == SPIN_ACCEPT_GREEDY) {          // greedy matching needs the arg-max only
        MaxArg best = {-INFINITY, 0x7fffffff};
        if (vec) {
            for (int i = g_lo + tid; i < g_hi; i += kStatThreads) {
                const float4 v = x4[i];
                best = better(best, MaxArg{v.x, 4 * i});
                best = better(best, MaxArg{v.y, 4 * i + 1});
                best = better(best, MaxArg{v.z, 4 * i + 2});
                best = better(best, MaxArg{v.w, 4 * i + 3});
            }
        } else {
            for (int i = e_lo + tid; i < e_hi; i += kStatThreads) best = better(best, MaxArg{x[i], i});
        }
        for (int off = 32; off > 0; off >>= 1) {
            MaxArg o = {__shfl_xor(best.v, off), __shfl_xor(best.i, off)};
            best = better(best, o);
        }
        if ((tid & 63) == 0) s_ma[tid >> 6] = best;
        __syncthreads();
        if (tid == 0) {
            best = s_ma[0];
            for (int w = 1; w < kStatThreads / 64; ++w) best = better(best, s_ma[w]);
            put_stats(P, out, best.v, 0.0, best.i);
        }
        return;
    }

    // Rejection sampling needs max and sum of exp(x - max).  One sweep: the exponentials are taken as they
    // are, exp(x), while the maximum is tracked beside them, and the sum is moved to the maximum at the end
    // (float64 has the range for that while the maximum lies within +-600; otherwise the row is swept
    // a second time against its maximum).  Logits below -700, minus infinity among them, count as -700:
    // less than 1e-43 of the largest term either way.
    s_tab[tid] = exp2((double)tid * (1.0 / 256.0));
    __syncthreads();
    float m = -INFINITY;
    double sum = 0.0, sum2 = 0.0;
    if (vec) {
        // kSweepLoads 16-byte loads per lane are issued before the first is used: with a few wavefronts per
        // SIMD the sweep is bound by the bytes it keeps in flight, not by its arithmetic.
        const int n4 = g_hi;
        for (int i0 = g_lo + tid; i0 < n4; i0 += kSweepLoads * kStatThreads) {
            float4 v[kSweepLoads];
#pragma unroll
            for (int j = 0; j < kSweepLoads; ++j) {
                const int i = i0 + j * kStatThreads;
                typedef __attribute__((ext_vector_type(4))) float f32x4_t;
                if (i >= n4) {
                    v[j] = float4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                } else if (STREAM) {
                    const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(x4 + i));
                    v[j] = float4{t[0], t[1], t[2], t[3]};
                } else {
                    v[j] = x4[i];
                }
            }
#pragma unroll
            for (int j = 0; j < kSweepLoads; ++j) {
                if (i0 + j * kStatThreads >= n4) break;
                m = fmaxf(m, fmaxf(fmaxf(v[j].x, v[j].y), fmaxf(v[j].z, v[j].w)));
                sum += exp_table64_in_range((double)fminf(fmaxf(v[j].x, -700.f), 700.f), s_tab);
                sum2 += exp_table64_in_range((double)fminf(fmaxf(v[j].y, -700.f), 700.f), s_tab);
                sum += exp_table64_in_range((double)fminf(fmaxf(v[j].z, -700.f), 700.f), s_tab);
                sum2 += exp_table64_in_range((double)fminf(fmaxf(v[j].w, -700.f), 700.f), s_tab);
            }
        }
    } else {
        for (int i = e_lo + tid; i < e_hi; i += kStatThreads) {
            m = fmaxf(m, x[i]);
            sum += exp_table64_in_range((double)fminf(fmaxf(x[i], -700.f), 700.f), s_tab);
        }
    }
    sum += sum2;
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((tid & 63) == 0) s_ref[tid >> 6] = m;
    __syncthreads();
    m = s_ref[0];
    for (int w = 1; w < kStatThreads / 64; ++w) m = fmaxf(m, s_ref[w]);
    const bool one_sweep = m >= -600.f && m <= 600.f;            // (the same decision in every lane)
    const double mx = (double)m;
    if (!one_sweep) {
        sum = 0.0;
        if (vec) {
            for (int i = g_lo + tid; i < g_hi; i += kStatThreads) {
                const float4 v = x4[i];
                sum += exp_table64((double)v.x - mx, s_tab) + exp_table64((double)v.y - mx, s_tab) +
                       exp_table64((double)v.z - mx, s_tab) + exp_table64((double)v.w - mx, s_tab);
            }
        } else {
            for (int i = e_lo + tid; i < e_hi; i += kStatThreads) sum += exp_table64((double)x[i] - mx, s_tab);
        }
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int w = 0; w < kStatThreads / 64; ++w) tot += s_sum[w];
        if (one_sweep) tot *= exp_table64_in_range(-mx, s_tab);
        put_stats(P, out, m, tot, 0);
    }
}

template <bool STREAM>
__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(AcceptParams P) {
    __shared__ StatShared sh;
    row_stats_body<STREAM>(P, blockIdx.x, sh);
}

// Logits of more than this many bytes are read with non-temporal loads: they do not fit the 256 MB last-level cache,
// where smaller batches are usually found right after the kernel that produced them (13b: 158 MB, 29 us with plain
// loads, 32 with non-temporal ones; 70b_gqa: 323 MB, 60 and 57).
constexpr int64_t kStreamLogitsBytes = 224ll << 20;
static bool stream_logits(const AcceptParams& p, int n_stat_rows) { return (int64_t)n_stat_rows * p.vocab * 4 > kStreamLogitsBytes; }

// The inverse CDF shared by the next-token kernels: the smallest id k with sum_{x<=k} mass(x) > u * total.
// The vocabulary is cut into blocks of 256 ids (a lane owns four consecutive ids of a block: 16-byte
// loads, consecutive lanes read consecutive memory); consecutive blocks form runs, the mass of every run
// is summed first, a scan over the run masses finds the run that holds u * total, and that run is computed
// once more and scanned inside.  The masses come from a source `src` with
//   src.load(x0, raw)     fetch what the four ids starting at x0 need (nothing beyond the vocabulary)
//   src.mass(x0, raw, m)  their masses (zero beyond the vocabulary)
struct DrawShared {
    double run[kMaxRuns];
    int last[16];
    double total, before;
    int cross;
};

// Second half of the search, by all threads of a workgroup: sh.run[0, n_runs) holds the run masses in id
// order, sh.last[0, n_last) the last id with mass of every part of the vocabulary (-1: none);
// run_blocks(run, b0, cnt) names the blocks of a run.  Wavefront 0 works, the others wait.  Returns false,
// with nothing written, when the total is not positive.
template <class Src, class RunBlocks>
__device__ __forceinline__ bool cdf_search(const Src& src, int V, double u, int32_t* out, DrawShared& sh, int n_runs,
                                           int n_last, RunBlocks run_blocks) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double* const s_run = sh.run;
    // wavefront 0 scans the run masses in id order: lane L takes a contiguous slice of them
    if (wave == 0) {
        const int per = (n_runs + 63) / 64;
        const int lo = min(n_runs, lane * per), hi = min(n_runs, lo + per);
        double mine = 0.0;
        for (int k = lo; k < hi; ++k) mine += s_run[k];
        double incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const double up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const double total = __shfl(incl, 63);
        const double thr = u * total;
        double excl = __shfl_up(incl, 1);
        if (lane == 0) excl = 0.0;
        if (lane == 0) {
            sh.total = total;
            sh.cross = -1;
        }
        // exactly the lanes where the running sum first passes the threshold look inside their slice
        if (incl > thr && !(excl > thr)) {
            double run = excl;
            int k = lo;
            for (; k < hi; ++k) {
                if (run + s_run[k] > thr) break;
                run += s_run[k];
            }
            if (k == hi) k = hi - 1;             // summation orders may differ in the last bit
            // several lanes can only get here when the sums are not monotone by rounding: lowest wins
            const unsigned long long who = __ballot(1);
            if (lane == __ffsll((long long)who) - 1) {
                sh.cross = k;
                sh.before = run;
            }
        }
    }
    __syncthreads();
    const double total = sh.total;
    if (!(total > 0.0)) {                    // nothing to draw from: the caller decides what else to use
        __syncthreads();
        return false;
    }
    const int cross = sh.cross;
    if (cross < 0) {                         // u'*Z at or beyond the total: last id with mass
        if (tid == 0) {
            int k = -1;
            for (int w = 0; w < n_last; ++w) k = max(k, sh.last[w]);
            *out = k >= 0 ? k : V - 1;
        }
        return true;
    }
    if (wave == 0) {
        const double thr = u * total;
        double before = sh.before;           // mass in front of the block at hand
        int lastpos = -1, b0 = 0, cnt = 0;
        run_blocks(cross, b0, cnt);
        bool found = false;
        for (int k = 0; k < cnt && !found; ++k) {
            const int x0 = (b0 + k) * 256 + 4 * lane;
            typename Src::Raw raw;
            src.load(x0, raw);
            double m[4];
            src.mass(x0, raw, m);
            const double mine = (m[0] + m[1]) + (m[2] + m[3]);
            double incl = mine;
            for (int off = 1; off < 64; off <<= 1) {
                const double up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            incl += before;
            double excl = __shfl_up(incl, 1);
            if (lane == 0) excl = before;
            const bool hit = incl > thr && !(excl > thr);
            int id = 0x7fffffff;
            if (hit) {
                double run = excl;
                id = -1;
                for (int j = 0; j < 4; ++j) {
                    run += m[j];
                    if (run > thr) { id = x0 + j; break; }
                }
                if (id < 0)
                    for (int j = 3; j >= 0 && id < 0; --j)
                        if (m[j] > 0.0) id = x0 + j;
                if (id < 0) id = min(x0, V - 1);
            }
            const unsigned long long who = __ballot(hit);
            if (who) {
                if (lane == __ffsll((long long)who) - 1) *out = id;
                found = true;
            }
            for (int j = 0; j < 4; ++j)
                if (m[j] > 0.0) lastpos = x0 + j;
            before = __shfl(incl, 63);
        }
        if (!found) {
            // the recomputed run fell short of its first sum by rounding: its last id with mass
            for (int off = 32; off > 0; off >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, off));
            if (lane == 0) *out = lastpos >= 0 ? lastpos : min(b0 * 256, V - 1);
        }
    }
    return true;
}

// Masses of `n_blocks` consecutive blocks starting at block `first`, by one wavefront: the loads of four
// blocks are issued before the first of them is used.  done(k, mass of block k as a wavefront-wide sum)
// is called for every block in turn; returns this lane's last id with mass (-1: none).
template <class Src, class Done>
__device__ __forceinline__ int wave_block_masses(const Src& src, int first, int n_blocks, Done done) {
    const int lane = threadIdx.x & 63;
    int last = -1;
    for (int b0 = 0; b0 < n_blocks; b0 += 4) {
        typename Src::Raw raw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (b0 + j < n_blocks) src.load((first + b0 + j) * 256 + 4 * lane, raw[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (b0 + j >= n_blocks) break;
            const int x0 = (first + b0 + j) * 256 + 4 * lane;
            double m[4];
            src.mass(x0, raw[j], m);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (m[e] > 0.0) last = x0 + e;
            done(b0 + j, (m[0] + m[1]) + (m[2] + m[3]));
        }
    }
    return last;
}

// The whole search by one workgroup of T threads: wavefront w owns a contiguous range of blocks, `rs`
// consecutive blocks of a wavefront form a run (rs = 1 up to 262144 ids at T = 256), so that runs in
// (wavefront, run) order are in id order.  Called by all threads of the workgroup.
template <int T, class Src>
__device__ __forceinline__ bool draw_inverse_cdf(const Src& src, int V, double u, int32_t* out, DrawShared& sh) {
    constexpr int kWaves = T / 64;
    constexpr int kRunsPerWave = kMaxRuns / kWaves;
    static_assert(kWaves <= 16 && kRunsPerWave >= 1, "workgroup size");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nb = (V + 255) >> 8;                           // blocks of 256 ids
    const int nbw = (nb + kWaves - 1) / kWaves;              // blocks per wavefront
    const int rs = (nbw + kRunsPerWave - 1) / kRunsPerWave;  // blocks per run
    const int rpw = (nbw + rs - 1) / rs;                     // runs per wavefront
    double acc = 0.0;
    int in_run = 0;
    int last = wave_block_masses(src, wave * nbw, nbw, [&](int k, double m) {
        acc += m;
        if (++in_run == rs || k == nbw - 1) {
            double run = acc;
            for (int off = 32; off > 0; off >>= 1) run += __shfl_xor(run, off);
            if (lane == 0) sh.run[wave * rpw + k / rs] = run;
            acc = 0.0;
            in_run = 0;
        }
    });
    for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off));
    if (lane == 0) sh.last[wave] = last;
    __syncthreads();
    return cdf_search(src, V, u, out, sh, rpw * kWaves, kWaves, [&](int run, int& b0, int& cnt) {
        const int w = run / rpw, r = run - w * rpw;
        b0 = w * nbw + r * rs;
        cnt = min(rs, nbw - r * rs);
    });
}

// Masses of the linear acceptance's next-token draw: the residual max(0, p - q) of the rejected row, or the
// target distribution p itself (bonus row, or p == q up to rounding).
struct ResidualSrc {
    const float* tl;
    const float* dl;
    double tmax, tinv, dmax, dinv;
    const double* tab;
    int V;
    bool use_residual, vec;
    struct Raw {
        float a[4], b[4];
    };
    __device__ __forceinline__ void load(int x0, Raw& r) const {
        for (int j = 0; j < 4; ++j) {
            r.a[j] = -INFINITY;
            r.b[j] = 0.f;
        }
        if (vec && x0 + 3 < V) {
            const float4 va = *reinterpret_cast<const float4*>(tl + x0);
            r.a[0] = va.x; r.a[1] = va.y; r.a[2] = va.z; r.a[3] = va.w;
            if (use_residual) {
                const float4 vb = *reinterpret_cast<const float4*>(dl + x0);
                r.b[0] = vb.x; r.b[1] = vb.y; r.b[2] = vb.z; r.b[3] = vb.w;
            }
        } else {
            for (int j = 0; j < 4; ++j)
                if (x0 + j < V) {
                    r.a[j] = tl[x0 + j];
                    if (use_residual) r.b[j] = dl[x0 + j];
                }
        }
    }
    __device__ __forceinline__ void mass(int x0, const Raw& r, double m[4]) const {
        for (int j = 0; j < 4; ++j) {
            double v = 0.0;
            if (x0 + j < V) {
                v = exp_table64((double)r.a[j] - tmax, tab) * tinv;
                if (use_residual) {
                    v -= exp_table64((double)r.b[j] - dmax, tab) * dinv;
                    v = v > 0.0 ? v : 0.0;
                }
            }
            m[j] = v;
        }
    }
};

// Row statistics written by other workgroups of the same launch are read past this CU's caches.
__device__ __forceinline__ float stat_max(const AcceptParams& P, int idx) {
    return __hip_atomic_load(P.row_max + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double stat_sum(const AcceptParams& P, int idx) {
    return __hip_atomic_load(P.row_sum + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t stat_arg(const AcceptParams& P, int idx) {
    return __hip_atomic_load(P.row_arg + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Maximum of a row and the sum of exp(x - maximum) over it.
__device__ __forceinline__ void row_stat(const AcceptParams& P, int row, double& mx, double& sum) {
    mx = (double)stat_max(P, row);
    sum = stat_sum(P, row);
}

// Row offsets that came from the device (the entry point that allocates nothing cannot read them on the
// host) are checked by the kernels: a request whose rows do not lie inside the tensors reports -1, -1.
__device__ __forceinline__ bool request_ok(const AcceptParams& P, int r0, int g) { return r0 >= 0 && g >= 1 && r0 + g <= P.n_rows; }

// The first-reject scan of one request once the statistics of its rows are known, by the workgroup's first
// wavefront (64 draft rows at a time, one per lane): writes n_accepted, and in greedy mode the next token;
// returns the accepted length in that wavefront's lanes (the caller passes it on through LDS).
__device__ __forceinline__ int first_reject(const AcceptParams& P, int req, int r0, int g, const double* tab) {
    const int lane = threadIdx.x & 63;
    const int base = r0 + req;                  // first target row of the request
    const int n_target = P.n_rows + P.n_req;
    const int V = P.vocab;
    int n = g;
    for (int t0 = 0; t0 < g; t0 += 64) {
        const int t = t0 + lane;
        bool keep = true;
        if (t < g) {
            const int d = P.draft_tokens[r0 + t];
            if (d < 0 || d >= V) {
                keep = false;               // a token outside the vocabulary is never kept
            } else if (P.mode == SPIN_ACCEPT_GREEDY) {
                keep = d == stat_arg(P, base + t);
            } else {
                double tm, ts, dm, ds;
                row_stat(P, base + t, tm, ts);
                row_stat(P, n_target + r0 + t, dm, ds);
                const double p = exp_table64((double)P.target_logits[(int64_t)(base + t) * V + d] - tm, tab) / ts;
                const double q = exp_table64((double)P.draft_logits[(int64_t)(r0 + t) * V + d] - dm, tab) / ds;
                keep = P.u_accept[r0 + t] * q < p;
            }
        }
        const unsigned long long rejected = __ballot(!keep);
        if (rejected) {
            n = t0 + __ffsll((long long)rejected) - 1;
            break;
        }
    }
    if (lane == 0) {
        P.n_accepted[req] = n;
        if (P.mode == SPIN_ACCEPT_GREEDY) P.next_token[req] = stat_arg(P, base + n);
    }
    return n;
}

// What the next token of a request with n accepted draft tokens is drawn from.
__device__ __forceinline__ ResidualSrc residual_src(const AcceptParams& P, int req, int r0, int g, int n, const double* tab) {
    const int base = r0 + req, n_target = P.n_rows + P.n_req, V = P.vocab;
    ResidualSrc src;
    src.tl = P.target_logits + (int64_t)(base + n) * V;
    double sum;
    row_stat(P, base + n, src.tmax, sum);
    src.tinv = 1.0 / sum;
    const bool residual = n < g;
    src.dl = residual ? P.draft_logits + (int64_t)(r0 + n) * V : src.tl;
    src.dmax = 0.0;
    src.dinv = 1.0;
    if (residual) {
        row_stat(P, n_target + r0 + n, src.dmax, sum);
        src.dinv = 1.0 / sum;
    }
    src.tab = tab;
    src.V = V;
    src.vec = (V % 4 == 0) && (((reinterpret_cast<uintptr_t>(src.tl) | reinterpret_cast<uintptr_t>(src.dl)) & 15) == 0);
    src.use_residual = residual;
    return src;
}

struct FinishShared {
    DrawShared draw;
    int n;
};

// The acceptance of one request by one workgroup of T threads once the statistics of its rows are known:
// the first-reject scan, then the next token -- arg-max (greedy), or the inverse CDF over the residual
// max(0, p - q) / the bonus row's p.  `tab` = 2^(j/256), filled and visible to all threads.
template <int T>
__device__ __forceinline__ void finish_request(const AcceptParams& P, int req, int r0, int g, FinishShared& sh, const double* tab) {
    if (!request_ok(P, r0, g)) {
        if (threadIdx.x == 0) {
            P.n_accepted[req] = -1;
            P.next_token[req] = -1;
        }
        return;
    }
    if (threadIdx.x < 64) {
        const int n = first_reject(P, req, r0, g, tab);
        if (threadIdx.x == 0) sh.n = n;
    }
    __syncthreads();
    if (P.mode == SPIN_ACCEPT_GREEDY) return;
    ResidualSrc src = residual_src(P, req, r0, g, sh.n, tab);
    for (int attempt = 0; attempt < 2; ++attempt) {
        if (draw_inverse_cdf<T>(src, P.vocab, P.u_sample[req], &P.next_token[req], sh.draw)) break;
        src.use_residual = false;                // p == q up to rounding: draw from p instead
    }
}

// One workgroup per request, after row_stats_kernel: greedy mode (the scan is all there is to do), vocabularies
// beyond the run table of accept_draw_kernel, and the entry point that allocates nothing.
constexpr int kFinishThreads = 1024;
__global__ __launch_bounds__(kFinishThreads) void accept_finish_kernel(AcceptParams P) {
    __shared__ FinishShared sh;
    __shared__ double s_tab[256];
    if (threadIdx.x < 256) s_tab[threadIdx.x] = exp2((double)threadIdx.x * (1.0 / 256.0));
    __syncthreads();
    const int r0 = P.row_off[blockIdx.x];
    finish_request<kFinishThreads>(P, blockIdx.x, r0, P.row_off[blockIdx.x + 1] - r0, sh, s_tab);
}

// Batches of up to kInlineReqs requests bring their row offsets in the kernel arguments (every workgroup
// needs two of them before it can start; from the argument segment they cost a scalar load).
constexpr int kInlineReqs = 959;
struct InlineOffsets {
    int32_t off[kInlineReqs + 1];
};

// Count this workgroup in on a request's counter; true in all its threads when it is the last of
// `expected`, in which case the counter is zero again.  Device-scope stores of this thread before the
// call have completed before the count moves (the wavefront waits for their acknowledgement), and the
// thread that sees the full count reads what the others wrote with device-scope loads issued after its
// atomic has returned: no cache is written back or invalidated as a whole.
__device__ __forceinline__ bool arrive_last(int32_t* counter, int expected, int* s_flag) {
    if (threadIdx.x == 0) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const int seen = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = seen == expected - 1;
        if (seen == expected - 1) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return *s_flag != 0;
}

// The whole acceptance in one launch, for small vocabularies (where a second launch would cost more than the
// next-token draw itself).  Workgroup (slot, request) takes the statistics of one logits row of the request --
// slots 0..g its target rows (the last one the bonus row), slots g+1..2g its draft rows (rejection mode) --
// then counts itself in on the request's arrival counter, and the workgroup that arrives last runs the
// request's first-reject scan and next-token draw.
template <bool INLINE>
__global__ __launch_bounds__(kStatThreads) void accept_small_kernel(AcceptParams P, InlineOffsets io) {
    __shared__ StatShared st;
    __shared__ FinishShared sh;
    __shared__ int s_is_last;
    const int req = blockIdx.y, slot = blockIdx.x;
    const int r0 = INLINE ? io.off[req] : P.row_off[req];
    const int g = (INLINE ? io.off[req + 1] : P.row_off[req + 1]) - r0;
    const int n_slots = P.mode == SPIN_ACCEPT_GREEDY ? g + 1 : 2 * g + 1;
    if (slot >= n_slots) return;
    const int n_target = P.n_rows + P.n_req;
    const int row = slot <= g ? r0 + req + slot : n_target + r0 + (slot - g - 1);
    row_stats_body(P, row, st);
    if (!arrive_last(P.arrive + req, n_slots, &s_is_last)) return;
    if (P.mode == SPIN_ACCEPT_GREEDY) st.tab[threadIdx.x] = 0.0;   // (not used; keeps the table defined)
    __syncthreads();
    finish_request<kStatThreads>(P, req, r0, g, sh, st.tab);
}

// Second launch (rejection mode, after row_stats_kernel): the next token of every request.  The vocabulary
// is cut into P.draw_parts <= kDrawChunks parts (as many as keep all workgroups of the launch resident at
// once); workgroup (part, request) runs the request's first-reject scan (every part
// for itself: a few rows, and cheaper than one more launch or a wait), sums the masses of its part's blocks
// of 256 ids into the request's run table, counts itself in on the request's arrival counter, and the
// workgroup that arrives last scans the table and looks inside the block that holds u' * Z.  The counter
// is zero before the launch and the last arrival puts it back to zero.
constexpr int kDrawChunks = 8;
constexpr int kDrawBlocks = 512;     // blocks of 256 ids per request in the run table: vocabularies up to 131072

template <bool INLINE>
__global__ __launch_bounds__(kStatThreads) void accept_draw_kernel(AcceptParams P, InlineOffsets io) {
    __shared__ DrawShared sh;
    __shared__ double s_tab[256];
    __shared__ int s_is_last;
    const int req = blockIdx.y, part = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = INLINE ? io.off[req] : P.row_off[req];
    const int g = (INLINE ? io.off[req + 1] : P.row_off[req + 1]) - r0;
    __shared__ int s_n;
    s_tab[tid] = exp2((double)tid * (1.0 / 256.0));
    __syncthreads();
    if (!request_ok(P, r0, g)) return;                          // (the whole workgroup, and all parts alike)
    if (tid < 64) {
        const int n_here = first_reject(P, req, r0, g, s_tab);  // (all parts write the same n_accepted)
        if (tid == 0) s_n = n_here;
    }
    __syncthreads();
    const int n = s_n;
    const int V = P.vocab;
    const int nb = (V + 255) >> 8;
    const int parts = P.draw_parts;
    const int nbp = (nb + parts - 1) / parts;                   // blocks per part
    const int nbw = (nbp + 3) / 4;                              // blocks per wavefront
    ResidualSrc src = residual_src(P, req, r0, g, n, s_tab);
    double* const runs = P.draw_runs + (int64_t)req * kDrawBlocks;
    int32_t* const lasts = P.draw_last + (int64_t)req * kDrawChunks;
    const int first = part * nbp + wave * nbw;
    const int cnt = max(0, min(min(nbw, nbp - wave * nbw), nb - first));
    int last = wave_block_masses(src, first, cnt, [&](int k, double m) {
        for (int off = 32; off > 0; off >>= 1) m += __shfl_xor(m, off);
        if (lane == 0) __hip_atomic_store(runs + first + k, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    });
    for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off));
    if (lane == 0) sh.last[wave] = last;
    // every wavefront's run masses must have completed before thread 0 moves the count
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kStatThreads / 64; ++w) last = max(last, sh.last[w]);
        __hip_atomic_store(lasts + part, last, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!arrive_last(P.arrive + req, parts, &s_is_last)) return;
    for (int k = tid; k < nb; k += kStatThreads) sh.run[k] = __hip_atomic_load(runs + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid < parts) sh.last[tid] = __hip_atomic_load(lasts + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (cdf_search(src, V, P.u_sample[req], &P.next_token[req], sh, nb, parts, [&](int run, int& b0, int& c) {
            b0 = run;
            c = 1;
        }))
        return;
    // the residual summed to zero (p == q up to rounding): this workgroup alone draws from p itself
    src.use_residual = false;
    draw_inverse_cdf<kStatThreads>(src, V, P.u_sample[req], &P.next_token[req], sh);
}

// Greedy verification of token trees: one wavefront per request, one lane per draft token (at most
// 64).  A token "matches" when it equals the arg-max of its parent's target row; the walk starts below
// the last prefix token and moves to the lowest-numbered matching child until there is none.
__global__ __launch_bounds__(64) void accept_tree_kernel(AcceptParams P, const int32_t* parent, int32_t* path) {
    const int req = blockIdx.x, lane = threadIdx.x;
    const int r0 = P.row_off[req];
    const int g = P.row_off[req + 1] - r0;
    const int base = r0 + req;                  // target row of the root; node t owns row base + 1 + t
    int par = -2;
    bool match = false;
    if (lane < g) {
        par = parent[r0 + lane];
        match = P.draft_tokens[r0 + lane] == P.row_arg[base + par + 1];
    }
    int cur = -1, n = 0;
    while (true) {
        const unsigned long long next = __ballot(match && par == cur);
        if (!next) break;
        cur = __ffsll((long long)next) - 1;
        if (lane == 0) path[r0 + n] = cur;
        ++n;
    }
    if (lane >= n && lane < g) path[r0 + lane] = -1;
    if (lane == 0) {
        P.n_accepted[req] = n;
        P.next_token[req] = P.row_arg[base + cur + 1];
    }
}

// Rejection-sampling verification of token trees: one workgroup per request walks down from the
// root.  At a node with target distribution p the children are tried in index order against what is
// left of p: with R_0 = p, s_0 = 1, child c (token d, drawn from q_c) is accepted iff
// u_c q_c(d) s_k < R_k(d); a rejected child gives R_{k+1} = max(0, R_k - s_k q_c), s_{k+1} = sum R_{k+1}
// (one sweep over the vocabulary by the whole workgroup; a child that would leave nothing is ignored).
// When no child is accepted the next token is drawn from R_k.  R_k(x) is never stored: it is
// re-evaluated from the k+1 logits rows involved, whose pointers and scale factors sit in LDS.
constexpr int kMaxSiblings = 64;

__global__ __launch_bounds__(kTreeThreads) void accept_tree_reject_kernel(AcceptParams P, const int32_t* parent,
                                                                          int32_t* path) {
    constexpr int kWaves = kTreeThreads / 64;
    __shared__ DrawShared sh;
    __shared__ double s_tab[256];
    __shared__ const float* s_row[kMaxSiblings];     // draft rows of the rejected children of the current node
    __shared__ double s_dmax[kMaxSiblings], s_coef[kMaxSiblings];   // their maxima and s_j / (their sums)
    __shared__ double s_part[kWaves];
    __shared__ int s_flag;
    const int req = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = P.row_off[req];
    const int g = P.row_off[req + 1] - r0;
    const int base = r0 + req;                  // target row of the root; node t owns row base + 1 + t
    const int n_target = P.n_rows + P.n_req;
    const int V = P.vocab;
    if (tid < 256) s_tab[tid] = exp2((double)tid * (1.0 / 256.0));
    __syncthreads();

    int cur = -1, n = 0;
    while (true) {
        const float* tl = P.target_logits + (int64_t)(base + cur + 1) * V;
        const double tmax = (double)P.row_max[base + cur + 1], tinv = 1.0 / P.row_sum[base + cur + 1];
        int k = 0;              // rejected children of this node that count
        double sk = 1.0;
        // R_depth(x) for one id
        auto mass1 = [&](int x, int depth) {
            double v = exp_table64((double)tl[x] - tmax, s_tab) * tinv;
            for (int j = 0; j < depth; ++j) {
                v -= exp_table64((double)s_row[j][x] - s_dmax[j], s_tab) * s_coef[j];
                v = v > 0.0 ? v : 0.0;
            }
            return v;
        };
        bool moved = false;
        for (int c = cur + 1; c < g; ++c) {         // children come after their parent
            if (parent[r0 + c] != cur) continue;
            const float* dl = P.draft_logits + (int64_t)(r0 + c) * V;
            const double dmax = (double)P.row_max[n_target + r0 + c], dinv = 1.0 / P.row_sum[n_target + r0 + c];
            if (tid == 0) {
                const int d = P.draft_tokens[r0 + c];
                bool keep = false;
                if (d >= 0 && d < V) {
                    const double q = exp_table64((double)dl[d] - dmax, s_tab) * dinv;
                    keep = P.u_accept[r0 + c] * q * sk < mass1(d, k);
                }
                s_flag = keep;
            }
            __syncthreads();
            const bool keep = s_flag;
            if (keep) {
                if (tid == 0) path[r0 + n] = c;
                cur = c;
                ++n;
                moved = true;
                __syncthreads();                     // s_flag is written again at the next node
                break;
            }
            // rejected: what would be left after taking s_k q_c out of R_k?
            if (k < kMaxSiblings) {
                if (tid == 0) {
                    s_row[k] = dl;
                    s_dmax[k] = dmax;
                    s_coef[k] = sk * dinv;
                }
                __syncthreads();
                double sum = 0.0;
                for (int x = tid; x < V; x += kTreeThreads) sum += mass1(x, k + 1);
                for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
                if (lane == 0) s_part[wave] = sum;
                __syncthreads();
                double tot = 0.0;
                for (int w = 0; w < kWaves; ++w) tot += s_part[w];
                if (tot > 0.0) {
                    ++k;
                    sk = tot;
                }
            }
            __syncthreads();
        }
        if (moved) continue;

        // ---- no child was accepted: the next token comes from R_k
        const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(tl) & 15) == 0) &&
                         ((reinterpret_cast<uintptr_t>(P.draft_logits) & 15) == 0);
        struct TreeSrc {
            const float* tl;
            const float* const* rows;
            const double *dmax, *coef, *tab;
            double tmax, tinv;
            int k, V;
            bool vec;
            struct Raw {
                float a[4];
            };
            __device__ __forceinline__ void load(int x0, Raw& r) const {
                for (int j = 0; j < 4; ++j) r.a[j] = -INFINITY;
                if (vec && x0 + 3 < V) {
                    const float4 va = *reinterpret_cast<const float4*>(tl + x0);
                    r.a[0] = va.x; r.a[1] = va.y; r.a[2] = va.z; r.a[3] = va.w;
                } else {
                    for (int j = 0; j < 4; ++j)
                        if (x0 + j < V) r.a[j] = tl[x0 + j];
                }
            }
            __device__ __forceinline__ void mass(int x0, const Raw& r, double m[4]) const {
                for (int j = 0; j < 4; ++j) m[j] = x0 + j < V ? exp_table64((double)r.a[j] - tmax, tab) * tinv : 0.0;
                for (int s = 0; s < k; ++s) {
                    float b[4] = {0.f, 0.f, 0.f, 0.f};
                    if (vec && x0 + 3 < V) {
                        const float4 vb = *reinterpret_cast<const float4*>(rows[s] + x0);
                        b[0] = vb.x; b[1] = vb.y; b[2] = vb.z; b[3] = vb.w;
                    } else {
                        for (int j = 0; j < 4; ++j)
                            if (x0 + j < V) b[j] = rows[s][x0 + j];
                    }
                    for (int j = 0; j < 4; ++j)
                        if (x0 + j < V) {
                            const double v = m[j] - exp_table64((double)b[j] - dmax[s], tab) * coef[s];
                            m[j] = v > 0.0 ? v : 0.0;
                        }
                }
            }
        };
        const TreeSrc src = {tl, s_row, s_dmax, s_coef, s_tab, tmax, tinv, k, V, vec};
        if (!draw_inverse_cdf<kTreeThreads>(src, V, P.u_sample[req], &P.next_token[req], sh)) {
            // cannot happen (R_0 sums to one and a child that leaves nothing is ignored); be defined anyway
            if (tid == 0) P.next_token[req] = P.row_arg[base + cur + 1];
        }
        break;
    }
    if (tid >= n && tid < g) path[r0 + tid] = -1;
    if (tid == 0) P.n_accepted[req] = n;
}

hipError_t launch_accept_tree(const AcceptParams& p, const int32_t* parent, int32_t* path, hipStream_t stream) {
    if (p.n_req <= 0) return hipSuccess;
    const int n_stat_rows = p.mode == SPIN_ACCEPT_GREEDY ? p.n_rows + p.n_req : 2 * p.n_rows + p.n_req;
    if (stream_logits(p, n_stat_rows)) hipLaunchKernelGGL(row_stats_kernel<true>, dim3(n_stat_rows), dim3(kStatThreads), 0, stream, p);
    else hipLaunchKernelGGL(row_stats_kernel<false>, dim3(n_stat_rows), dim3(kStatThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.mode == SPIN_ACCEPT_GREEDY)
        hipLaunchKernelGGL(accept_tree_kernel, dim3(p.n_req), dim3(64), 0, stream, p, parent, path);
    else
        hipLaunchKernelGGL(accept_tree_reject_kernel, dim3(p.n_req), dim3(kTreeThreads), 0, stream, p, parent, path);
    return hipGetLastError();
}

// Vocabularies up to this size are handled in one launch.
constexpr int kSmallVocab = 8192;

// The path launch_accept takes: one launch (0), row statistics + spread draw (1), row statistics + one workgroup
// per request (2).  Only the last reads the row offsets from memory when the host's copy of them is at hand.
static int accept_path(const AcceptParams& p, int max_draft) {
    const bool counters = p.arrive && p.n_req <= 65535;
    if (counters && max_draft >= 1 && p.vocab <= kSmallVocab) return 0;
    if (counters && p.mode == SPIN_ACCEPT_REJECTION && p.vocab <= kDrawBlocks * 256 && p.draw_runs && p.draw_last) return 1;
    return 2;
}

bool accept_reads_row_off(const AcceptParams& p, int max_draft) {
    return p.n_req > kInlineReqs || accept_path(p, max_draft) == 2;
}

hipError_t launch_accept(const AcceptParams& p, int max_draft, const int32_t* row_off_host, hipStream_t stream, LaunchTiming* timing) {
    if (timing) timing->second = false;
    if (p.n_req <= 0) return hipSuccess;
    const int path = accept_path(p, max_draft);
    hipEvent_t t0 = timing ? timing->ev[0] : nullptr, t1 = timing ? timing->ev[1] : nullptr;
    hipEvent_t t2 = timing ? timing->ev[2] : nullptr, t3 = timing ? timing->ev[3] : nullptr;
    const bool inl = row_off_host && p.n_req <= kInlineReqs;
    if (!inl && !p.row_off) return hipErrorInvalidValue;
    InlineOffsets io;
    io.off[0] = 0;
    if (inl) memcpy(io.off, row_off_host, (size_t)(p.n_req + 1) * 4);
    const dim3 block(kStatThreads);
    hipError_t e;
    if (path == 0) {
        const int slots = p.mode == SPIN_ACCEPT_GREEDY ? max_draft + 1 : 2 * max_draft + 1;
        const dim3 grid(slots, p.n_req);
        if (inl) hipExtLaunchKernelGGL(accept_small_kernel<true>, grid, block, 0, stream, t0, t1, 0, p, io);
        else hipExtLaunchKernelGGL(accept_small_kernel<false>, grid, block, 0, stream, t0, t1, 0, p, io);
        return hipGetLastError();
    }
    const int n_stat_rows = p.mode == SPIN_ACCEPT_GREEDY ? p.n_rows + p.n_req : 2 * p.n_rows + p.n_req;
    if (stream_logits(p, n_stat_rows)) hipExtLaunchKernelGGL(row_stats_kernel<true>, dim3(n_stat_rows), block, 0, stream, t0, t1, 0, p);
    else hipExtLaunchKernelGGL(row_stats_kernel<false>, dim3(n_stat_rows), block, 0, stream, t0, t1, 0, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (path == 1) {
        // as many parts per request as keep every workgroup of the launch resident at once: a second round of
        // workgroups would double the length of what is a chain of dependent memory round trips
        static std::atomic<int> resident{0};
        int res = resident.load();
        if (res == 0) {
            int per_cu = 0, dev = 0, cus = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, accept_draw_kernel<true>, kStatThreads, 0) != hipSuccess ||
                hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
                return hipErrorUnknown;
            res = std::max(1, per_cu * cus);
            resident.store(res);
        }
        AcceptParams pd = p;
        pd.draw_parts = std::max(1, std::min(kDrawChunks, res / p.n_req));
        const dim3 dgrid(pd.draw_parts, p.n_req);
        if (inl) hipExtLaunchKernelGGL(accept_draw_kernel<true>, dgrid, block, 0, stream, t2, t3, 0, pd, io);
        else hipExtLaunchKernelGGL(accept_draw_kernel<false>, dgrid, block, 0, stream, t2, t3, 0, pd, io);
    } else {
        if (!p.row_off) return hipErrorInvalidValue;
        hipExtLaunchKernelGGL(accept_finish_kernel, dim3(p.n_req), dim3(kFinishThreads), 0, stream, t2, t3, 0, p);
    }
    e = hipGetLastError();
    if (e == hipSuccess && timing) timing->second = true;
    return e;
}

size_t accept_draw_scratch_bytes(int64_t n_req, size_t* last_bytes) {
    *last_bytes = (size_t)n_req * kDrawChunks * 4;
    return (size_t)n_req * kDrawBlocks * 8;
}

}  // namespace spin

// ------------------------------------------------------------------------------------------------
// spin_accept for callers that cannot allocate (HIP graph capture, serving loops and harnesses that
// forbid hipMalloc): the same two kernels, with the row statistics in a file-scope device array
// instead of a context's workspace.  Every GPU holds its own copy of the array at its own address;
// the address is looked up once per device and only that pointer is ever handed to HIP calls.
namespace {

constexpr int kStaticRows = SPIN_NOALLOC_MAX_STAT_ROWS;
// per statistics row: float64 sum | float max | int32 arg-max
static __device__ __align__(256) unsigned char scratch[(size_t)kStaticRows * 16];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each GPU, null until looked up
std::mutex g_scratch_mutex;

// Device address of the scratch array on the current device (looked up on the first call per device).
hipError_t static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

namespace spin {
hipError_t resolve_static_scratch() {
    void* p = nullptr;
    return static_scratch(&p);
}
}  // namespace spin

extern "C" int spin_accept_noalloc(int32_t mode, int32_t n_req, int32_t n_rows, const int32_t* q_offset_dev,
                                   const int32_t* draft_tokens_dev, const float* target_logits_dev,
                                   const float* draft_logits_dev, int32_t vocab, const double* u_accept_dev,
                                   const double* u_sample_dev, int32_t* n_accepted_dev, int32_t* next_token_dev,
                                   void* hip_stream) {
    if (mode != SPIN_ACCEPT_GREEDY && mode != SPIN_ACCEPT_REJECTION) return SPIN_EINVAL;
    if (n_req < 0 || n_rows < 0 || vocab < 1) return SPIN_EINVAL;
    if (vocab > spin::kMaxVocab) return SPIN_EUNSUPPORTED;
    if (n_req == 0) return SPIN_OK;
    if (n_rows < n_req) return SPIN_EINVAL;               // every request brings at least one draft token
    if (2 * (int64_t)n_rows + n_req > kStaticRows) return SPIN_ENOSPC;
    if (!q_offset_dev || !draft_tokens_dev || !target_logits_dev || !n_accepted_dev || !next_token_dev) return SPIN_EINVAL;
    if (mode == SPIN_ACCEPT_REJECTION && (!draft_logits_dev || !u_accept_dev || !u_sample_dev)) return SPIN_EINVAL;
    void* base = nullptr;
    if (static_scratch(&base) != hipSuccess) return SPIN_EHIP;
    spin::AcceptParams p = {};
    p.row_off = q_offset_dev;
    p.draft_tokens = draft_tokens_dev;
    p.target_logits = target_logits_dev;
    p.draft_logits = draft_logits_dev;
    p.u_accept = u_accept_dev;
    p.u_sample = u_sample_dev;
    p.row_sum = (double*)base;
    p.row_max = (float*)((char*)base + (size_t)kStaticRows * 8);
    p.row_arg = (int32_t*)((char*)base + (size_t)kStaticRows * 12);
    p.n_accepted = n_accepted_dev;
    p.next_token = next_token_dev;
    p.n_req = n_req;
    p.n_rows = n_rows;
    p.vocab = vocab;
    p.mode = mode;
    return spin::launch_accept(p, 0, nullptr, (hipStream_t)hip_stream, nullptr) == hipSuccess ? SPIN_OK : SPIN_EHIP;
}
