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

#include "spin_device.h"

namespace spin {

constexpr int kStatThreads = 256;
constexpr int kFinishThreads = 256;

struct MaxArg {
    float v;
    int32_t i;
};

__device__ __forceinline__ MaxArg better(MaxArg a, MaxArg b) {
    // larger value wins; equal values -> lower index
    if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
    return a;
}

__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(AcceptParams P) {
    __shared__ MaxArg s_ma[kStatThreads / 64];
    __shared__ double s_sum[kStatThreads / 64];
    const int row = blockIdx.x;
    const int n_target = P.n_rows + P.n_req;
    const float* x = row < n_target ? P.target_logits + (int64_t)row * P.vocab
                                    : P.draft_logits + (int64_t)(row - n_target) * P.vocab;
    const int V = P.vocab;
    const int tid = threadIdx.x;
    const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);

    MaxArg best = {-INFINITY, 0x7fffffff};
    if (vec) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
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
    best = s_ma[0];
    for (int w = 1; w < kStatThreads / 64; ++w) best = better(best, s_ma[w]);

    if (P.mode == SPIN_ACCEPT_GREEDY) {          // greedy matching needs the arg-max only
        if (tid == 0) {
            P.row_max[row] = best.v;
            P.row_sum[row] = 0.0;
            P.row_arg[row] = best.i;
        }
        return;
    }
    const double mx = (double)best.v;
    double sum = 0.0;
    if (vec) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
        for (int i = tid; i < V / 4; i += kStatThreads) {
            const float4 v = x4[i];
            sum += exp((double)v.x - mx) + exp((double)v.y - mx) + exp((double)v.z - mx) + exp((double)v.w - mx);
        }
    } else {
        for (int i = tid; i < V; i += kStatThreads) sum += exp((double)x[i] - mx);
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int w = 0; w < kStatThreads / 64; ++w) tot += s_sum[w];
        P.row_max[row] = best.v;
        P.row_sum[row] = tot;
        P.row_arg[row] = best.i;
    }
}

__global__ __launch_bounds__(kFinishThreads) void accept_finish_kernel(AcceptParams P) {
    __shared__ int s_n;
    __shared__ double s_scan[kFinishThreads];
    __shared__ int s_last[kFinishThreads];
    __shared__ int s_hit;
    const int req = blockIdx.x;
    const int tid = threadIdx.x;
    const int r0 = P.row_off[req];
    const int g = P.row_off[req + 1] - r0;
    const int base = r0 + req;                  // first target row of the request
    const int n_target = P.n_rows + P.n_req;
    const int V = P.vocab;

    if (tid == 0) {
        int n = 0;
        for (; n < g; ++n) {
            const int d = P.draft_tokens[r0 + n];
            if (d < 0 || d >= V) break;         // a token outside the vocabulary is never kept
            if (P.mode == SPIN_ACCEPT_GREEDY) {
                if (d != P.row_arg[base + n]) break;
            } else {
                const double p = exp((double)P.target_logits[(int64_t)(base + n) * V + d] - (double)P.row_max[base + n]) /
                                 P.row_sum[base + n];
                const int dr = n_target + r0 + n;
                const double q = exp((double)P.draft_logits[(int64_t)(r0 + n) * V + d] - (double)P.row_max[dr]) /
                                 P.row_sum[dr];
                if (!(P.u_accept[r0 + n] * q < p)) break;
            }
        }
        s_n = n;
        P.n_accepted[req] = n;
        if (P.mode == SPIN_ACCEPT_GREEDY) P.next_token[req] = P.row_arg[base + n];
    }
    __syncthreads();
    if (P.mode == SPIN_ACCEPT_GREEDY) return;

    const int n = s_n;
    const float* tl = P.target_logits + (int64_t)(base + n) * V;
    const double tmax = (double)P.row_max[base + n], tsum = P.row_sum[base + n];
    const bool residual = n < g;
    const float* dl = residual ? P.draft_logits + (int64_t)(r0 + n) * V : nullptr;
    const double dmax = residual ? (double)P.row_max[n_target + r0 + n] : 0.0;
    const double dsum = residual ? P.row_sum[n_target + r0 + n] : 1.0;

    // thread t owns the contiguous id range [lo, hi)
    const int per = (V + kFinishThreads - 1) / kFinishThreads;
    const int lo = min(V, tid * per), hi = min(V, lo + per);
    bool use_residual = residual;
    for (int attempt = 0; attempt < 2; ++attempt) {
        auto mass = [&](int x) -> double {
            const double p = exp((double)tl[x] - tmax) / tsum;
            if (!use_residual) return p;
            const double q = exp((double)dl[x] - dmax) / dsum;
            const double r = p - q;
            return r > 0.0 ? r : 0.0;
        };
        double seg = 0.0;
        int last = -1;
        for (int x = lo; x < hi; ++x) {
            const double m = mass(x);
            seg += m;
            if (m > 0.0) last = x;
        }
        s_scan[tid] = seg;
        s_last[tid] = last;
        if (tid == 0) s_hit = -1;
        __syncthreads();
        // inclusive scan over the 256 segment sums (Hillis-Steele, float64)
        for (int off = 1; off < kFinishThreads; off <<= 1) {
            const double add = tid >= off ? s_scan[tid - off] : 0.0;
            __syncthreads();
            s_scan[tid] += add;
            __syncthreads();
        }
        const double total = s_scan[kFinishThreads - 1];
        if (use_residual && !(total > 0.0)) {   // p == q up to rounding: draw from p instead
            use_residual = false;
            __syncthreads();
            continue;
        }
        const double thr = P.u_sample[req] * total;
        const double incl = s_scan[tid];
        const double excl = tid > 0 ? s_scan[tid - 1] : 0.0;
        // the first segment whose inclusive sum passes the threshold holds the answer
        if (incl > thr && !(excl > thr)) {
            double run = excl;
            int k = -1;
            for (int x = lo; x < hi; ++x) {
                run += mass(x);
                if (run > thr) { k = x; break; }
            }
            // run may fall short of incl by rounding of the two summation orders
            if (k < 0) k = last >= 0 ? last : hi - 1;
            s_hit = k;
        }
        __syncthreads();
        if (tid == 0) {
            int k = s_hit;
            if (k < 0) {                         // u'*Z at or beyond the total: last id with mass
                for (int t = kFinishThreads - 1; t >= 0 && k < 0; --t) k = s_last[t];
                if (k < 0) k = V - 1;
            }
            P.next_token[req] = k;
        }
        break;
    }
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
