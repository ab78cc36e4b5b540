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

#include <mutex>

#include "spin_device.h"

namespace spin {

constexpr int kStatThreads = 256;
constexpr int kFinishThreads = 1024;
constexpr int kMaxRuns = 4096;   // (step, wavefront) runs of 256 ids kept in LDS: vocabularies up to 1M ids

struct MaxArg {
    float v;
    int32_t i;
};

__device__ __forceinline__ MaxArg better(MaxArg a, MaxArg b) {
    // larger value wins; equal values -> lower index
    if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
    return a;
}

// exp(d) in float64 for the sums and masses, d below about 700: d = (256 e + j) ln2/256 + r with
// |r| <= ln2/512, so exp(d) = 2^e * 2^(j/256) * exp(r) with a 256-entry table (in LDS) and a cubic for
// exp(r) (remainder r^4/24 < 1.4e-13 relative, the rounded ln2/256 adds 2.4e-14: four orders below what
// the accept decisions need, and about half the float64 instructions of the general routine).  Minus infinity (and anything below
// -800) gives 0.
__device__ __forceinline__ double exp_table64(double d, const double* tab) {
    d = fmax(d, -800.0);
    const double kd = __builtin_rint(d * 369.3299304675746);            // 256 / ln 2
    const double r = fma(kd, -0.0027076061740622863, d);                     // ln2/256 rounded: off by 9.1e-20, |kd| < 3e5
    const int k = (int)kd;
    double p = fma(r, 1.0 / 6.0, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(tab[k & 255] * p, k >> 8);
}

__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(AcceptParams P) {
    __shared__ MaxArg s_ma[kStatThreads / 64];
    __shared__ double s_sum[kStatThreads / 64];
    __shared__ float s_ref[kStatThreads / 64];
    __shared__ double s_tab[256];
    const int row = blockIdx.x;
    const int n_target = P.n_rows + P.n_req;
    const float* x = row < n_target ? P.target_logits + (int64_t)row * P.vocab
                                    : P.draft_logits + (int64_t)(row - n_target) * P.vocab;
    const int V = P.vocab;
    const int tid = threadIdx.x;
    const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
    const float4* x4 = reinterpret_cast<const float4*>(x);

    if (P.mode == SPIN_ACCEPT_GREEDY) {          // greedy matching needs the arg-max only
        MaxArg best = {-INFINITY, 0x7fffffff};
        if (vec) {
            for (int i = tid; i < V / 4; i += kStatThreads) {
                const float4 v = x4[i];
                best = better(best, MaxArg{v.x, 4 * i});
                best = better(best, MaxArg{v.y, 4 * i + 1});
                best = better(best, MaxArg{v.z, 4 * i + 2});
                best = better(best, MaxArg{v.w, 4 * i + 3});
            }
        } else {
            for (int i = tid; i < V; i += kStatThreads) best = better(best, MaxArg{x[i], i});
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
            P.row_max[row] = best.v;
            P.row_sum[row] = 0.0;
            P.row_arg[row] = best.i;
        }
        return;
    }

    // Rejection sampling needs max and sum of exp(x - max).  One sweep: the exponentials are taken
    // against a reference found in the row's first elements while the true maximum is tracked beside
    // them, and the sum is moved to the true maximum at the end (float64 has the range for that as
    // long as the two are within a few hundred of each other; otherwise the row is swept twice).
    s_tab[tid] = exp2((double)tid * (1.0 / 256.0));
    float ref = -INFINITY;
    if (vec) {
        if (tid < V / 4) {
            const float4 v = x4[tid];
            ref = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
        }
    } else if (tid < V) {
        ref = x[tid];
    }
    for (int off = 32; off > 0; off >>= 1) ref = fmaxf(ref, __shfl_xor(ref, off));
    if ((tid & 63) == 0) s_ref[tid >> 6] = ref;
    __syncthreads();
    ref = s_ref[0];
    for (int w = 1; w < kStatThreads / 64; ++w) ref = fmaxf(ref, s_ref[w]);
    bool one_sweep = ref > -INFINITY && ref < INFINITY;

    float m = -INFINITY;
    double sum = 0.0;
    if (one_sweep) {
        const double rd = (double)ref;
        if (vec) {
#pragma unroll 2                                   // two loads in flight per lane (measured: 40 -> 36 us on the 13B batch)
            for (int i = tid; i < V / 4; i += kStatThreads) {
                const float4 v = x4[i];
                m = fmaxf(m, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
                sum += exp_table64((double)v.x - rd, s_tab) + exp_table64((double)v.y - rd, s_tab) +
                       exp_table64((double)v.z - rd, s_tab) + exp_table64((double)v.w - rd, s_tab);
            }
        } else {
            for (int i = tid; i < V; i += kStatThreads) {
                m = fmaxf(m, x[i]);
                sum += exp_table64((double)x[i] - rd, s_tab);
            }
        }
    } else {
        if (vec) {
            for (int i = tid; i < V / 4; i += kStatThreads) {
                const float4 v = x4[i];
                m = fmaxf(m, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
            }
        } else {
            for (int i = tid; i < V; i += kStatThreads) m = fmaxf(m, x[i]);
        }
    }
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    __syncthreads();                               // s_ref is reused for the maximum
    if ((tid & 63) == 0) s_ref[tid >> 6] = m;
    __syncthreads();
    m = s_ref[0];
    for (int w = 1; w < kStatThreads / 64; ++w) m = fmaxf(m, s_ref[w]);
    if (one_sweep && !(m - ref < 500.f)) one_sweep = false;     // (the same decision in every lane)
    const double mx = (double)m;
    if (!one_sweep) {
        sum = 0.0;
        if (vec) {
            for (int i = tid; i < V / 4; i += kStatThreads) {
                const float4 v = x4[i];
                sum += exp((double)v.x - mx) + exp((double)v.y - mx) + exp((double)v.z - mx) + exp((double)v.w - mx);
            }
        } else {
            for (int i = tid; i < V; i += kStatThreads) sum += exp((double)x[i] - mx);
        }
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int w = 0; w < kStatThreads / 64; ++w) tot += s_sum[w];
        if (one_sweep) tot *= exp((double)ref - mx);
        P.row_max[row] = m;
        P.row_sum[row] = tot;
        P.row_arg[row] = 0;
    }
}

// The inverse CDF shared by the next-token kernels: the smallest id k with sum_{x<=k} mass(x) > u * total.
// mass4(x0, m) gives the masses of the four ids starting at x0 (zero beyond the vocabulary).  The
// vocabulary is walked in steps of 4 * kFinishThreads ids; in a step thread t owns the four ids
// step*4T + 4t .. +3 (16-byte loads, consecutive lanes read consecutive memory), so wavefront w owns a
// contiguous run of 256 ids.  Pass 1 leaves the mass of every (step, wavefront) run in LDS; a scan over
// those finds the run that holds u * total; its wavefront recomputes the run and scans inside it.
// Called by all threads of the workgroup; returns false, with nothing written, when the total is not positive.
struct DrawShared {
    double* run;      // [kMaxRuns]
    int* last;        // [kFinishThreads / 64]
    double* total;
    double* before;
    int* cross;
};

template <class Mass4>
__device__ __forceinline__ bool draw_inverse_cdf(Mass4 mass4, int V, double u, int32_t* out, const DrawShared& sh) {
    constexpr int kWaves = kFinishThreads / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_steps = (V + 4 * kFinishThreads - 1) / (4 * kFinishThreads);
    const int n_runs = n_steps * kWaves;
    double* const s_run = sh.run;
    int* const s_last = sh.last;
    double& s_total = *sh.total;
    double& s_before = *sh.before;
    int& s_cross = *sh.cross;
    int last = -1;
    for (int st = 0; st < n_steps; ++st) {
        const int x0 = st * 4 * kFinishThreads + 4 * tid;
        double m[4];
        mass4(x0, m);
        double run = (m[0] + m[1]) + (m[2] + m[3]);
        for (int j = 0; j < 4; ++j)
            if (m[j] > 0.0) last = x0 + j;
        for (int off = 32; off > 0; off >>= 1) run += __shfl_xor(run, off);
        if (lane == 0) s_run[st * kWaves + wave] = run;
    }
    for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off));
    if (lane == 0) s_last[wave] = last;
    __syncthreads();
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
            s_total = total;
            s_cross = -1;
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
                s_cross = k;
                s_before = run;
            }
        }
    }
    __syncthreads();
    const double total = s_total;
    if (!(total > 0.0)) {                    // nothing to draw from: the caller decides what else to use
        __syncthreads();
        return false;
    }
    const int cross = s_cross;
    if (cross < 0) {                         // u'*Z at or beyond the total: last id with mass
        if (tid == 0) {
            int k = -1;
            for (int w = 0; w < kWaves; ++w) k = max(k, s_last[w]);
            *out = k >= 0 ? k : V - 1;
        }
        return true;
    }
    if (wave == cross % kWaves) {
        const int x0 = (cross / kWaves) * 4 * kFinishThreads + 4 * tid;
        const double thr = u * total;
        double m[4];
        mass4(x0, m);
        const double mine = (m[0] + m[1]) + (m[2] + m[3]);
        double incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const double up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        incl += s_before;
        double excl = __shfl_up(incl, 1);
        if (lane == 0) excl = s_before;
        const bool hit = incl > thr && !(excl > thr);
        int k = 0x7fffffff;
        if (hit) {
            double run = excl;
            k = -1;
            for (int j = 0; j < 4; ++j) {
                run += m[j];
                if (run > thr) { k = x0 + j; break; }
            }
            if (k < 0)
                for (int j = 3; j >= 0 && k < 0; --j)
                    if (m[j] > 0.0) k = x0 + j;
            if (k < 0) k = min(x0, V - 1);
        }
        const unsigned long long who = __ballot(hit);
        if (who) {
            if (lane == __ffsll((long long)who) - 1) *out = k;
        } else {
            // the recomputed run fell short of its first sum by rounding: its last id with mass
            int lastpos = -1;
            for (int j = 0; j < 4; ++j)
                if (m[j] > 0.0) lastpos = x0 + j;
            for (int off = 32; off > 0; off >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, off));
            if (lane == 0) *out = lastpos >= 0 ? lastpos : min(x0, V - 1);
        }
    }
    return true;
}

__global__ __launch_bounds__(kFinishThreads) void accept_finish_kernel(AcceptParams P) {
    constexpr int kWaves = kFinishThreads / 64;
    __shared__ int s_n;
    __shared__ double s_run[kMaxRuns];
    __shared__ int s_last[kWaves];
    __shared__ double s_total, s_before;
    __shared__ int s_cross;
    __shared__ double s_tab[256];                 // 2^(j/256) for exp_table64
    const DrawShared sh = {s_run, s_last, &s_total, &s_before, &s_cross};
    const int req = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = P.row_off[req];
    const int g = P.row_off[req + 1] - r0;
    const int base = r0 + req;                  // first target row of the request
    const int n_target = P.n_rows + P.n_req;
    const int V = P.vocab;
    // Row offsets that came from the device (the entry point that allocates nothing cannot read them on
    // the host) are checked here: a request whose rows do not lie inside the tensors reports -1, -1.
    if (r0 < 0 || g < 1 || r0 + g > P.n_rows) {
        if (tid == 0) {
            P.n_accepted[req] = -1;
            P.next_token[req] = -1;
        }
        return;
    }

    if (tid < 256) s_tab[tid] = exp2((double)tid * (1.0 / 256.0));   // ready at the barrier below
    // ---- first-reject scan: wavefront 0 tests 64 draft rows at a time, one per lane
    if (wave == 0) {
        int n = g;
        for (int t0 = 0; t0 < g; t0 += 64) {
            const int t = t0 + lane;
            bool keep = true;
            if (t < g) {
                const int d = P.draft_tokens[r0 + t];
                if (d < 0 || d >= V) {
                    keep = false;               // a token outside the vocabulary is never kept
                } else if (P.mode == SPIN_ACCEPT_GREEDY) {
                    keep = d == P.row_arg[base + t];
                } else {
                    const double p = exp((double)P.target_logits[(int64_t)(base + t) * V + d] - (double)P.row_max[base + t]) /
                                     P.row_sum[base + t];
                    const int dr = n_target + r0 + t;
                    const double q = exp((double)P.draft_logits[(int64_t)(r0 + t) * V + d] - (double)P.row_max[dr]) /
                                     P.row_sum[dr];
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
            s_n = n;
            P.n_accepted[req] = n;
            if (P.mode == SPIN_ACCEPT_GREEDY) P.next_token[req] = P.row_arg[base + n];
        }
    }
    __syncthreads();
    if (P.mode == SPIN_ACCEPT_GREEDY) return;

    // ---- next token: inverse CDF over the residual max(0, p - q), or over the bonus row's p
    const int n = s_n;
    const float* tl = P.target_logits + (int64_t)(base + n) * V;
    const double tmax = (double)P.row_max[base + n], tinv = 1.0 / P.row_sum[base + n];
    const bool residual = n < g;
    const float* dl = residual ? P.draft_logits + (int64_t)(r0 + n) * V : tl;
    const double dmax = residual ? (double)P.row_max[n_target + r0 + n] : 0.0;
    const double dinv = residual ? 1.0 / P.row_sum[n_target + r0 + n] : 1.0;
    const bool vec = (V % 4 == 0) && (((reinterpret_cast<uintptr_t>(tl) | reinterpret_cast<uintptr_t>(dl)) & 15) == 0);

    bool use_residual = residual;
    for (int attempt = 0; attempt < 2; ++attempt) {
        // masses of the four ids starting at x0 (zero beyond the vocabulary)
        auto mass4 = [&](int x0, double m[4]) {
            float a[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY}, b[4] = {0.f, 0.f, 0.f, 0.f};
            if (vec && x0 + 3 < V) {
                const float4 va = *reinterpret_cast<const float4*>(tl + x0);
                a[0] = va.x; a[1] = va.y; a[2] = va.z; a[3] = va.w;
                if (use_residual) {
                    const float4 vb = *reinterpret_cast<const float4*>(dl + x0);
                    b[0] = vb.x; b[1] = vb.y; b[2] = vb.z; b[3] = vb.w;
                }
            } else {
                for (int j = 0; j < 4; ++j)
                    if (x0 + j < V) {
                        a[j] = tl[x0 + j];
                        if (use_residual) b[j] = dl[x0 + j];
                    }
            }
            for (int j = 0; j < 4; ++j) {
                double v = 0.0;
                if (x0 + j < V) {
                    v = exp_table64((double)a[j] - tmax, s_tab) * tinv;
                    if (use_residual) {
                        v -= exp_table64((double)b[j] - dmax, s_tab) * dinv;
                        v = v > 0.0 ? v : 0.0;
                    }
                }
                m[j] = v;
            }
        };
        if (draw_inverse_cdf(mass4, V, P.u_sample[req], &P.next_token[req], sh)) break;
        use_residual = false;                    // p == q up to rounding: draw from p instead
    }
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

__global__ __launch_bounds__(kFinishThreads) void accept_tree_reject_kernel(AcceptParams P, const int32_t* parent,
                                                                            int32_t* path) {
    constexpr int kWaves = kFinishThreads / 64;
    __shared__ double s_run[kMaxRuns];
    __shared__ int s_last[kWaves];
    __shared__ double s_total, s_before;
    __shared__ int s_cross;
    __shared__ double s_tab[256];
    __shared__ const float* s_row[kMaxSiblings];     // draft rows of the rejected children of the current node
    __shared__ double s_dmax[kMaxSiblings], s_coef[kMaxSiblings];   // their maxima and s_j / (their sums)
    __shared__ double s_part[kWaves];
    __shared__ int s_flag;
    const DrawShared sh = {s_run, s_last, &s_total, &s_before, &s_cross};
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
                for (int x = tid; x < V; x += kFinishThreads) sum += mass1(x, k + 1);
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
        auto mass4 = [&](int x0, double m[4]) {
            float a[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (vec && x0 + 3 < V) {
                const float4 va = *reinterpret_cast<const float4*>(tl + x0);
                a[0] = va.x; a[1] = va.y; a[2] = va.z; a[3] = va.w;
            } else {
                for (int j = 0; j < 4; ++j)
                    if (x0 + j < V) a[j] = tl[x0 + j];
            }
            for (int j = 0; j < 4; ++j) m[j] = x0 + j < V ? exp_table64((double)a[j] - tmax, s_tab) * tinv : 0.0;
            for (int s = 0; s < k; ++s) {
                float b[4] = {0.f, 0.f, 0.f, 0.f};
                if (vec && x0 + 3 < V) {
                    const float4 vb = *reinterpret_cast<const float4*>(s_row[s] + x0);
                    b[0] = vb.x; b[1] = vb.y; b[2] = vb.z; b[3] = vb.w;
                } else {
                    for (int j = 0; j < 4; ++j)
                        if (x0 + j < V) b[j] = s_row[s][x0 + j];
                }
                for (int j = 0; j < 4; ++j)
                    if (x0 + j < V) {
                        const double v = m[j] - exp_table64((double)b[j] - s_dmax[s], s_tab) * s_coef[s];
                        m[j] = v > 0.0 ? v : 0.0;
                    }
            }
        };
        if (!draw_inverse_cdf(mass4, V, P.u_sample[req], &P.next_token[req], sh)) {
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
    hipLaunchKernelGGL(row_stats_kernel, dim3(n_stat_rows), dim3(kStatThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.mode == SPIN_ACCEPT_GREEDY)
        hipLaunchKernelGGL(accept_tree_kernel, dim3(p.n_req), dim3(64), 0, stream, p, parent, path);
    else
        hipLaunchKernelGGL(accept_tree_reject_kernel, dim3(p.n_req), dim3(kFinishThreads), 0, stream, p, parent, path);
    return hipGetLastError();
}

hipError_t launch_accept(const AcceptParams& p, hipStream_t stream, hipEvent_t ev_mid) {
    const int n_stat_rows = p.mode == SPIN_ACCEPT_GREEDY ? p.n_rows + p.n_req : 2 * p.n_rows + p.n_req;
    if (n_stat_rows > 0) {
        hipLaunchKernelGGL(row_stats_kernel, dim3(n_stat_rows), dim3(kStatThreads), 0, stream, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (ev_mid) {
        hipError_t e = hipEventRecord(ev_mid, stream);
        if (e != hipSuccess) return e;
    }
    if (p.n_req > 0) {
        hipLaunchKernelGGL(accept_finish_kernel, dim3(p.n_req), dim3(kFinishThreads), 0, stream, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
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
    return spin::launch_accept(p, (hipStream_t)hip_stream, nullptr) == hipSuccess ? SPIN_OK : SPIN_EHIP;
}
