// Speculative sampling on the device: softmax statistics of logit rows, the accept
// test u * D(d) < T(d), the residual max(0, T - D) and the fixed-point inverse-CDF
// sampler that draws the replacement / bonus token (and the draft's own samples).
//
// Fixed-point sampler: w(x) = floor(r(x) * 2^32) as 64-bit integers, S = sum w (integer,
// so independent of the reduction tree), threshold = floor(k_u * S / 2^24) with
// k_u = u * 2^24, result = first x whose inclusive running sum exceeds the threshold.
// Every decision after the float32 probabilities is integer arithmetic, which is what
// makes the result reproducible bit for bit by any other implementation.
#include "launch.h"

namespace spd {

constexpr int kSampThreads = 1024;

struct RowStats { float mx; float sum; int argmax; int pad; };

// Numerator of the softmax: exp((l - max) / temp) through the hardware exponential (relative
// error about |argument| * 6e-8).  Statistics, accept test, residual and the draft's D row all
// use this one function, so the probabilities of a row are consistent with its sum.
__device__ __forceinline__ float softmax_num(float l, float mx, float inv_temp) { return __expf((l - mx) * inv_temp); }

__device__ __forceinline__ unsigned long long shfl_up_u64(unsigned long long v, int off) {
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_up(lo, off);
    hi = __shfl_up(hi, off);
    return ((unsigned long long)hi << 32) | lo;
}

// Exclusive prefix sum of one value per thread over the whole workgroup (1024 threads);
// *total receives the workgroup sum.  `tmp` = 17 x u64 of shared memory.
__device__ unsigned long long block_exclusive_scan(unsigned long long v, unsigned long long *tmp,
                                                   unsigned long long *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    unsigned long long incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        unsigned long long t = shfl_up_u64(incl, off);
        if (lane >= off) incl += t;
    }
    __syncthreads();                      // tmp may still be in use by a previous call
    if (lane == 63) tmp[w] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long run = 0;
        for (int i = 0; i < kSampThreads / 64; ++i) { unsigned long long t = tmp[i]; tmp[i] = run; run += t; }
        tmp[16] = run;
    }
    __syncthreads();
    *total = tmp[16];
    return tmp[w] + incl - v;
}

// floor(r * 2^32) for r >= 0: the scale is exact (a power of two).  Below 1 -- every probability except an
// exact 1 -- the result fits 32 bits and one truncating conversion instruction gives it; the general
// float -> 64-bit conversion (a long instruction sequence) is only needed for r >= 1.
__device__ __forceinline__ unsigned long long fixed_weight(float r) {
    const float scaled = r * 4294967296.0f;
    if (__builtin_expect(r >= 1.0f, 0)) return (unsigned long long)scaled;
    return (unsigned long long)__float2uint_rz(scaled);
}

__device__ __forceinline__ unsigned long long threshold_of(float u, unsigned long long S) {
    unsigned long long k_u = (unsigned long long)(u * 16777216.0f);   // u is a multiple of 2^-24
    unsigned long long hi = __umul64hi(k_u, S), lo = k_u * S;
    return (hi << 40) | (lo >> 24);                           // floor(k_u * S / 2^24), 128-bit product
}

// Draw from the distribution proportional to r(x), x in [0, V).  Returns -1 if every
// weight truncates to zero.  All threads of the workgroup must call it; all get the result.
template <class F>
__device__ int sample_inverse_cdf(F r, int V, float u, unsigned long long *tmp, int *result) {
    const int C = (V + kSampThreads - 1) / kSampThreads;
    const int x0 = min(V, (int)threadIdx.x * C), x1 = min(V, x0 + C);
    unsigned long long part = 0;
    for (int x = x0; x < x1; ++x) part += fixed_weight(r(x));
    unsigned long long S;
    unsigned long long excl = block_exclusive_scan(part, tmp, &S);
    if (threadIdx.x == 0) *result = -1;
    __syncthreads();
    if (S != 0) {
        unsigned long long thr = threshold_of(u, S);
        if (excl <= thr && thr < excl + part) {               // exactly one thread
            unsigned long long run = excl;
            for (int x = x0; x < x1; ++x) {
                run += fixed_weight(r(x));
                if (run > thr) { *result = x; break; }
            }
        }
    }
    __syncthreads();
    return *result;
}

// ---------------------------------------------------------------------------------
// softmax statistics of logit rows: max, argmax (lowest index), sum exp((l - max) / temp)
// ---------------------------------------------------------------------------------
__device__ void row_stats(const float *__restrict__ row, int V, float inv_temp, RowStats *out_shared) {
    // out_shared: one RowStats in shared memory, valid after the call for all threads
    __shared__ float s_mx[kSampThreads / 64];
    __shared__ int s_arg[kSampThreads / 64];
    __shared__ float s_sum[kSampThreads / 64];
    float mx = -INFINITY;
    int arg = 0x7fffffff;
    for (int x = threadIdx.x; x < V; x += blockDim.x) {
        float v = row[x];
        if (v > mx) { mx = v; arg = x; }                       // strided: first hit is the lowest index
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float om = __shfl_xor(mx, off);
        int oa = __shfl_xor(arg, off);
        if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if (lane == 0) { s_mx[w] = mx; s_arg[w] = arg; }
    __syncthreads();
    mx = s_mx[0]; arg = s_arg[0];
    for (int i = 1; i < nw; ++i)
        if (s_mx[i] > mx || (s_mx[i] == mx && s_arg[i] < arg)) { mx = s_mx[i]; arg = s_arg[i]; }
    float sum = 0.f;
    for (int x = threadIdx.x; x < V; x += blockDim.x) sum += softmax_num(row[x], mx, inv_temp);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) s_sum[w] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int i = 0; i < nw; ++i) t += s_sum[i];
        out_shared->mx = mx; out_shared->sum = t; out_shared->argmax = arg; out_shared->pad = 0;
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------
// Register-staged fast path: rows of up to 32768 entries (a multiple of 4, 16-byte aligned)
// are read exactly once, with coalesced 16-byte loads that are all in flight together:
// thread t holds float4 number i * 1024 + t of the row, i < kRowVec.  The generic code above
// (any vocabulary size) walks the row with dependent loads and is several times slower.
// ---------------------------------------------------------------------------------
constexpr int kRowVec = 8;

__device__ __forceinline__ bool row_fits_registers(const float *row, int V) {
    return (V & 3) == 0 && V <= kRowVec * kSampThreads * 4 && (reinterpret_cast<uintptr_t>(row) & 15) == 0;
}

// entries beyond the row read as `fill`
__device__ __forceinline__ void load_row(const float *__restrict__ row, int V, float fill, float4 (&v)[kRowVec]) {
    const int n4 = V >> 2;
#pragma unroll
    for (int i = 0; i < kRowVec; ++i) {
        const int q = i * kSampThreads + (int)threadIdx.x;
        v[i] = q < n4 ? reinterpret_cast<const float4 *>(row)[q] : float4{fill, fill, fill, fill};
    }
}

// softmax statistics from a row held in registers (same definition as row_stats)
__device__ void row_stats_regs(const float4 (&v)[kRowVec], int V, float inv_temp, RowStats *out_shared) {
    __shared__ float s_mx[kSampThreads / 64];
    __shared__ int s_arg[kSampThreads / 64];
    __shared__ float s_sum[kSampThreads / 64];
    float mx = -INFINITY;
    int arg = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < kRowVec; ++i) {                       // ascending x within the thread
        const int x0 = 4 * (i * kSampThreads + (int)threadIdx.x);
        const float e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e[j] > mx) { mx = e[j]; arg = x0 + j; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float om = __shfl_xor(mx, off);
        int oa = __shfl_xor(arg, off);
        if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) { s_mx[w] = mx; s_arg[w] = arg; }
    __syncthreads();
    static_assert(kSampThreads / 64 == 16, "the cross-wave steps below combine 16 partials in 16 lanes");
    mx = s_mx[lane & 15]; arg = s_arg[lane & 15];             // 16 wave results, combined by every 16-lane group
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) {
        float om = __shfl_xor(mx, off);
        int oa = __shfl_xor(arg, off);
        if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kRowVec; ++i) {                       // padding is -inf: exp gives 0
        sum += softmax_num(v[i].x, mx, inv_temp);
        sum += softmax_num(v[i].y, mx, inv_temp);
        sum += softmax_num(v[i].z, mx, inv_temp);
        sum += softmax_num(v[i].w, mx, inv_temp);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) s_sum[w] = sum;
    __syncthreads();
    float t = s_sum[lane & 15];                               // fixed tree over the 16 wave sums
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) t += __shfl_xor(t, off);
    if (threadIdx.x == 0) { out_shared->mx = mx; out_shared->sum = t; out_shared->argmax = arg; out_shared->pad = 0; }
    __syncthreads();
}

// Inverse-CDF draw (same definition as sample_inverse_cdf) from weights given per register
// slot: wf(i, j, x) = fixed-point weight of entry x = 4 (i * 1024 + t) + j.  The running sum
// over x is: all of slice i' < i, then the threads before t in slice i, then entries before j.
template <class WF>
__device__ int sample_inverse_cdf_regs(WF wf, int V, float u, unsigned long long *tmp, int *result) {
    // tmp: kRowVec * 17 u64 of shared memory
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // per slice: the sum of the thread's 4 weights, and its inclusive scan over the wave
    unsigned long long part[kRowVec], incl[kRowVec];
#pragma unroll
    for (int i = 0; i < kRowVec; ++i) {
        const int x0 = 4 * (i * kSampThreads + (int)threadIdx.x);
        unsigned long long p = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) p += (x0 + j < V) ? wf(i, j, x0 + j) : 0ull;
        part[i] = p;
        incl[i] = p;
    }
#pragma unroll
    for (int i = 0; i < kRowVec; ++i) {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            unsigned long long t = shfl_up_u64(incl[i], off);
            if (lane >= off) incl[i] += t;
        }
    }
    __syncthreads();                                          // tmp may still be in use by a previous call
    if (lane == 63) {
#pragma unroll
        for (int i = 0; i < kRowVec; ++i) tmp[i * 17 + w] = incl[i];
    }
    __syncthreads();
    // exclusive scan of the kRowVec x 16 wave totals (slices in order, waves in order) by wave 0:
    // two neighbouring entries per lane, integer sums, so the order of combination does not matter
    static_assert(kRowVec * (kSampThreads / 64) == 128, "one wave, two entries per lane");
    if (w == 0) {
        const int n0 = 2 * lane, n1 = 2 * lane + 1;
        const int a0 = (n0 >> 4) * 17 + (n0 & 15), a1 = (n1 >> 4) * 17 + (n1 & 15);
        const unsigned long long v0 = tmp[a0], v1 = tmp[a1];
        unsigned long long inc = v0 + v1;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            unsigned long long t = shfl_up_u64(inc, off);
            if (lane >= off) inc += t;
        }
        const unsigned long long excl = inc - v0 - v1;
        tmp[a0] = excl;
        tmp[a1] = excl + v0;
        if (lane == 63) { tmp[16] = inc; *result = -1; }      // slot 16 of slice 0 is free: the grand total
    }
    __syncthreads();
    const unsigned long long S = tmp[16];
    if (S != 0) {
        const unsigned long long thr = threshold_of(u, S);
#pragma unroll
        for (int i = 0; i < kRowVec; ++i) {
            const unsigned long long excl = tmp[i * 17 + w] + incl[i] - part[i];
            if (excl <= thr && thr < excl + part[i]) {        // exactly one (thread, slice)
                const int x0 = 4 * (i * kSampThreads + (int)threadIdx.x);
                unsigned long long run = excl;
                int found = -1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (x0 + j < V) run += wf(i, j, x0 + j);
                    if (found < 0 && run > thr) found = x0 + j;
                }
                *result = found;
            }
        }
    }
    __syncthreads();
    return *result;
}

__global__ __launch_bounds__(kSampThreads) void accept_stats_kernel(AcceptArgs a) {
    // one workgroup per logits row: target rows first, then draft rows
    const int n_t = a.n_seqs * (a.gamma + 1);
    const int r = blockIdx.x;
    const bool is_t = r < n_t;
    if (is_t && (a.flags & 1u)) return;
    if (!is_t && (a.flags & 2u)) return;
    const float *row = is_t ? a.target + (size_t)r * a.vocab : a.draft + (size_t)(r - n_t) * a.vocab;
    const float inv_temp = a.temperature > 0.f ? 1.0f / a.temperature : 1.0f;
    __shared__ RowStats st;
    if (row_fits_registers(row, a.vocab)) {
        float4 v[kRowVec];
        load_row(row, a.vocab, -INFINITY, v);
        row_stats_regs(v, a.vocab, inv_temp, &st);
    } else {
        row_stats(row, a.vocab, inv_temp, &st);
    }
    if (threadIdx.x == 0) reinterpret_cast<RowStats *>(a.stats)[r] = st;
}

// probability of token x in a row given its statistics (or the row itself if it holds probabilities)
struct RowProb {
    const float *row;
    RowStats st;
    float inv_temp;
    float inv_sum;      // 1 / st.sum (one exact division per row, one multiply per entry)
    int mode;           // 0 probabilities, 1 softmax of logits, 2 greedy one-hot
    __device__ __forceinline__ float operator()(int x) const { return of(row[x], x); }
    // probability of token x whose row entry is `value`
    __device__ __forceinline__ float of(float value, int x) const {
        if (mode == 0) return value;
        if (mode == 2) return x == st.argmax ? 1.0f : 0.0f;
        return softmax_num(value, st.mx, inv_temp) * inv_sum;
    }
};

__global__ __launch_bounds__(kSampThreads) void accept_decide_kernel(AcceptArgs a) {
    const int seq = blockIdx.x, G = a.gamma, V = a.vocab;
    const int n_t = a.n_seqs * (G + 1);
    const RowStats *stats = reinterpret_cast<const RowStats *>(a.stats);
    const float inv_temp = a.temperature > 0.f ? 1.0f / a.temperature : 1.0f;
    const int t_mode = (a.flags & 1u) ? 0 : (a.temperature > 0.f ? 1 : 2);
    const int d_mode = (a.flags & 2u) ? 0 : (a.temperature > 0.f ? 1 : 2);
    __shared__ int s_acc[64];
    __shared__ int s_k;
    __shared__ unsigned long long tmp[kRowVec * 17];
    __shared__ int result;

    auto t_row = [&](int j) {
        RowProb p;
        p.row = a.target + ((size_t)seq * (G + 1) + j) * V;
        p.st = t_mode == 0 ? RowStats{0.f, 1.f, 0, 0} : stats[seq * (G + 1) + j];
        p.inv_temp = inv_temp; p.mode = t_mode; p.inv_sum = 1.0f / p.st.sum;
        return p;
    };
    auto d_row = [&](int j) {
        RowProb p;
        p.row = a.draft + ((size_t)seq * G + j) * V;
        p.st = d_mode == 0 ? RowStats{0.f, 1.f, 0, 0} : stats[n_t + seq * G + j];
        p.inv_temp = inv_temp; p.mode = d_mode; p.inv_sum = 1.0f / p.st.sum;
        return p;
    };

    // accept tests: u_j * D_j(d_j) < T_j(d_j), one float32 multiply and one compare
    if ((int)threadIdx.x < G) {
        int j = threadIdx.x;
        int d = min(max(a.draft_tokens[(size_t)seq * a.token_stride + j], 0), V - 1);   // never index outside the row
        float Tx = t_row(j)(d), Dx = d_row(j)(d);
        float u = a.u[seq * (G + 1) + j];
        s_acc[j] = (__fmul_rn(u, Dx) < Tx) ? 1 : 0;
        if (a.accept_prob) {
            float ap = (Dx == 0.f) ? (Tx > 0.f ? 1.0f : 0.0f) : fminf(1.0f, Tx / Dx);
            a.accept_prob[seq * G + j] = ap;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int k = 0;
        while (k < G && s_acc[k]) ++k;
        s_k = k;
    }
    __syncthreads();
    const int k = s_k;

    int y;
    const float u_last = a.u[seq * (G + 1) + G];
    const RowProb T = t_row(k < G ? k : G);
    if (row_fits_registers(T.row, V) && (k == G || row_fits_registers(d_row(k).row, V))) {
        // rows once through registers; padding entries give probability 0 in every mode
        // (the distribution to draw from, as float32 probabilities, replaces the row in its registers)
        float4 tv[kRowVec];
        load_row(T.row, V, T.mode == 0 ? 0.f : -INFINITY, tv);
        if (k < G) {
            const RowProb D = d_row(k);
            const int n4 = V >> 2;
            const float fill = D.mode == 0 ? 0.f : -INFINITY;
#pragma unroll
            for (int i = 0; i < kRowVec; ++i) {               // the draft row passes through 4 registers at a time
                const int q = i * kSampThreads + (int)threadIdx.x;
                const int x0 = 4 * q;
                const float4 dq = q < n4 ? reinterpret_cast<const float4 *>(D.row)[q] : float4{fill, fill, fill, fill};
                tv[i].x = fmaxf(0.0f, __fsub_rn(T.of(tv[i].x, x0), D.of(dq.x, x0)));
                tv[i].y = fmaxf(0.0f, __fsub_rn(T.of(tv[i].y, x0 + 1), D.of(dq.y, x0 + 1)));
                tv[i].z = fmaxf(0.0f, __fsub_rn(T.of(tv[i].z, x0 + 2), D.of(dq.z, x0 + 2)));
                tv[i].w = fmaxf(0.0f, __fsub_rn(T.of(tv[i].w, x0 + 3), D.of(dq.w, x0 + 3)));
            }
        } else {
#pragma unroll
            for (int i = 0; i < kRowVec; ++i) {
                const int x0 = 4 * (i * kSampThreads + (int)threadIdx.x);
                tv[i] = float4{T.of(tv[i].x, x0), T.of(tv[i].y, x0 + 1), T.of(tv[i].z, x0 + 2), T.of(tv[i].w, x0 + 3)};
            }
        }
        auto elem = [](const float4 &q, int j) { return j == 0 ? q.x : (j == 1 ? q.y : (j == 2 ? q.z : q.w)); };
        y = sample_inverse_cdf_regs([&](int i, int j, int) { return fixed_weight(elem(tv[i], j)); }, V, u_last, tmp, &result);
        if (y < 0 && k < G) y = sample_inverse_cdf(T, V, u_last, tmp, &result);   // residual mass truncates to zero: rare
    } else if (k < G) {
        const RowProb D = d_row(k);
        y = sample_inverse_cdf([&](int x) { return fmaxf(0.0f, __fsub_rn(T(x), D(x))); }, V, u_last, tmp, &result);
        if (y < 0) y = sample_inverse_cdf(T, V, u_last, tmp, &result);
    } else {
        y = sample_inverse_cdf(T, V, u_last, tmp, &result);
    }
    if (threadIdx.x == 0) {
        a.n_accepted[seq] = k;
        a.next_token[seq] = y < 0 ? 0 : y;
    }
}

size_t accept_workspace_bytes(int n_seqs, int gamma) {
    return (size_t)n_seqs * (2 * gamma + 1) * sizeof(RowStats);
}

hipError_t launch_accept(const AcceptArgs &a, hipStream_t stream) {
    if (a.gamma < 1 || a.gamma > 63) return hipErrorInvalidValue;
    const bool need_stats = ((a.flags & 3u) != 3u);
    if (need_stats) {
        int n_rows = a.n_seqs * (2 * a.gamma + 1);
        hipLaunchKernelGGL(accept_stats_kernel, dim3(n_rows), dim3(kSampThreads), 0, stream, a);
    }
    hipLaunchKernelGGL(accept_decide_kernel, dim3(a.n_seqs), dim3(kSampThreads), 0, stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// draft step tail: D row = softmax(logits / temp) written out, one token drawn from it
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kSampThreads) void softmax_sample_kernel(const float *__restrict__ logits,
                                                                       size_t row_stride, int V,
                                                                       float temperature,
                                                                       const float *__restrict__ u, int u_stride,
                                                                       float *__restrict__ probs_out, size_t probs_stride,
                                                                       int32_t *__restrict__ token_out, int token_stride) {
    const int seq = blockIdx.x;
    const float *row = logits + (size_t)seq * row_stride;
    float *out = probs_out + (size_t)seq * probs_stride;
    const float u_seq = u[(size_t)seq * u_stride];
    __shared__ RowStats st;
    __shared__ unsigned long long tmp[kRowVec * 17];
    __shared__ int result;
    const float inv_temp = temperature > 0.f ? 1.0f / temperature : 1.0f;
    RowProb p;
    p.row = row; p.inv_temp = inv_temp; p.mode = temperature > 0.f ? 1 : 2;
    int y;
    if (row_fits_registers(row, V) && row_fits_registers(out, V)) {
        float4 v[kRowVec];
        load_row(row, V, -INFINITY, v);
        row_stats_regs(v, V, inv_temp, &st);
        p.st = st; p.inv_sum = 1.0f / st.sum;
        const int n4 = V >> 2;
#pragma unroll
        for (int i = 0; i < kRowVec; ++i) {
            const int q = i * kSampThreads + (int)threadIdx.x;
            const int x0 = 4 * q;
            v[i] = float4{p.of(v[i].x, x0), p.of(v[i].y, x0 + 1), p.of(v[i].z, x0 + 2), p.of(v[i].w, x0 + 3)};
            if (q < n4) reinterpret_cast<float4 *>(out)[q] = v[i];
        }
        auto elem = [](const float4 &q, int j) { return j == 0 ? q.x : (j == 1 ? q.y : (j == 2 ? q.z : q.w)); };
        y = sample_inverse_cdf_regs([&](int i, int j, int) { return fixed_weight(elem(v[i], j)); }, V, u_seq, tmp, &result);
    } else {
        row_stats(row, V, inv_temp, &st);
        p.st = st; p.inv_sum = 1.0f / st.sum;
        for (int x = threadIdx.x; x < V; x += blockDim.x) out[x] = p(x);
        y = sample_inverse_cdf(p, V, u_seq, tmp, &result);
    }
    if (threadIdx.x == 0) token_out[(size_t)seq * token_stride] = y < 0 ? 0 : y;
}

hipError_t launch_softmax_sample(const float *logits, size_t row_stride, int n_seqs, int vocab,
                                 float temperature, const float *u, int u_stride, float *probs_out,
                                 size_t probs_stride, int32_t *token_out, int token_stride, hipStream_t stream) {
    hipLaunchKernelGGL(softmax_sample_kernel, dim3(n_seqs), dim3(kSampThreads), 0, stream, logits,
                       row_stride, vocab, temperature, u, u_stride, probs_out, probs_stride, token_out, token_stride);
    return hipGetLastError();
}

}  // namespace spd
