// tree_accept kernels for gfx950: vocabulary-wide softmax statistics, the sibling chains of the
// draft rules, and the acceptance walk with the final inverse-CDF draw.
//
// What is computed follows Section 2 (steps 3-4: ordered acceptance, corrected distribution on the
// first rejection; tree form: longest accepted path) and Section 4 (temperature 0 = greedy) of the
// paper; the min(1, p/q) test and the positive-part residual are the speculative-sampling rule of
// the literature cited there.
//
// Decomposition (all bandwidth-bound, plain ALUs, 64-wide wave reductions):
//   1. accept_stats_kernel   every logits row is cut into ranges; one workgroup reduces one range
//                            to (max, argmax, sum exp) with fp32 loads and fp64 accumulation.
//                            The same workgroups pick every child's token logit out of its parent's row
//                            while that row is passing through them.
//   2. accept_chain_kernel   draft rules only.  A node's accept test depends only on its parent's two
//                            rows and on its rank among its siblings (as if all earlier siblings were
//                            rejected), so every parent is processed independently: a group of workgroups
//                            per parent walks its children in order and needs one vocabulary-wide
//                            reduction (the corrected law's normaliser) per child; the per-slice shares of
//                            every child's reduction stay in the workspace.
//   3. accept_walk_kernel    one workgroup per sequence, no waiting on anybody: the (cheap, LDS-only) walk
//                            from the root, then the final inverse-CDF draw.  The mass of the final law in
//                            every piece of the vocabulary is already known - from the ranges of step 1
//                            (minus the rejected tokens) or from the shares of step 2 - so only the piece that
//                            holds the crossing of the uniform is read again.
#include <atomic>

#include "tv_internal.hpp"

// No fused multiply-adds formed across expressions in this file: a share of a reduction rebuilt by another workgroup
// (accept_chain_kernel) must come out with the owner's bits whatever shape the surrounding code has.
#pragma clang fp contract(off)

namespace tv {

namespace {

constexpr int kStatThreads = 256;
constexpr int kChainThreads = 256;
constexpr int kChainWaves = kChainThreads / kWave;
constexpr int kDrawThreads = 1024;
constexpr int kDrawWaves = kDrawThreads / kWave;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// exp((z - m) / temperature) as the kernels evaluate it everywhere: fp32 exponent, fp64 afterwards.  A logit of
// -infinity (a banned token, a padded tail) has no mass; so has every entry while the reference m itself is still
// -infinity (nothing finite seen yet).
__device__ __forceinline__ double unnorm_prob(float z, float m, float it_log2e) {
    return (m == -INFINITY) ? 0.0 : (double)fast_exp2((z - m) * it_log2e);
}
// 1 / s for a row (or law) sum; a row without any mass gives every entry probability 0
__device__ __forceinline__ double inv_mass(double s) { return (s > 0.0) ? 1.0 / s : 0.0; }

// exp((m_old - m_new) / temperature), m_new >= m_old: the factor that carries a sum over to a higher reference.  The
// fp32 exponential (relative error ~1e-7, like every entry's own term) - the fp64 library routine is a long
// instruction sequence that would sit at the end of every workgroup of the statistics pass.
__device__ __forceinline__ double rescale_factor(float m_old, float m_new, float it_log2e) {
    return (double)fast_exp2((m_old - m_new) * it_log2e);
}

struct Red {          // (max, lowest argmax, sum exp relative to max)
    float m;
    int am;
    double s;
};

template <bool kGreedy>
__device__ __forceinline__ void red_push(Red& r, float z, int v, float it_log2e) {
    if (z > r.m) {
        if (!kGreedy && r.s != 0.0) r.s *= rescale_factor(r.m, z, it_log2e);
        r.m = z;
        r.am = v;
    }
    if (!kGreedy) r.s += unnorm_prob(z, r.m, it_log2e);
}

template <bool kGreedy>
__device__ __forceinline__ void red_push4(Red& r, const float4 x, int v0, float it) {
    const float mx = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
    if (mx > r.m) {
        if (!kGreedy && r.s != 0.0) r.s *= rescale_factor(r.m, mx, it);
        r.m = mx;
        r.am = (x.x == mx) ? v0 : (x.y == mx) ? v0 + 1 : (x.z == mx) ? v0 + 2 : v0 + 3;
    }
    if (!kGreedy) {
        r.s += unnorm_prob(x.x, r.m, it);
        r.s += unnorm_prob(x.y, r.m, it);
        r.s += unnorm_prob(x.z, r.m, it);
        r.s += unnorm_prob(x.w, r.m, it);
    }
}

// A batch of quads held in registers, quads in increasing vocabulary order (quad k starts at entry v0[k]; k
// with live[k] false holds nothing): the running maximum is raised once for the whole batch, so the fp64 rescale
// of the running sum - a long instruction sequence that a wave executes whenever any of its lanes needs it -
// runs once per batch, not once per quad.
template <bool kGreedy, int N>
__device__ __forceinline__ void red_push_batch(Red& r, const float4 (&x)[N], const int (&v0)[N], const bool (&live)[N],
                                               float it) {
    float bm = -INFINITY;
    int bam = 0x7fffffff;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float mx = fmaxf(fmaxf(x[k].x, x[k].y), fmaxf(x[k].z, x[k].w));
        if (live[k] && mx > bm) {            // strictly greater: the lowest index wins ties
            bm = mx;
            bam = (x[k].x == mx) ? v0[k] : (x[k].y == mx) ? v0[k] + 1 : (x[k].z == mx) ? v0[k] + 2 : v0[k] + 3;
        }
    }
    if (bm > r.m) {
        if (!kGreedy && r.s != 0.0) r.s *= rescale_factor(r.m, bm, it);
        r.m = bm;
        r.am = bam;
    }
    if (!kGreedy) {
#pragma unroll
        for (int k = 0; k < N; ++k)
            if (live[k]) {
                r.s += unnorm_prob(x[k].x, r.m, it);
                r.s += unnorm_prob(x[k].y, r.m, it);
                r.s += unnorm_prob(x[k].z, r.m, it);
                r.s += unnorm_prob(x[k].w, r.m, it);
            }
    }
}

__device__ __forceinline__ bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// One row of a logits matrix: fp32 elements, or bf16 (the upper half of the fp32 with the same value).
struct Row {
    const void* p;
    bool bf16;
    __device__ __forceinline__ float operator[](int v) const {
        return bf16 ? __uint_as_float((unsigned)static_cast<const unsigned short*>(p)[v] << 16)
                    : static_cast<const float*>(p)[v];
    }
    // entries 4k .. 4k+3 can be fetched with one load (16 bytes of fp32, 8 bytes of bf16)
    __device__ __forceinline__ bool quad_aligned() const {
        return (reinterpret_cast<uintptr_t>(p) & (bf16 ? 7 : 15)) == 0;
    }
};
__device__ __forceinline__ Row logits_row(const AcceptArgs& a, const void* mat, int b, int node) {
    const int64_t e = ((int64_t)b * a.T + node) * a.row_stride;
    return Row{static_cast<const unsigned char*>(mat) + e * (a.logits_bf16 ? 2 : 4), a.logits_bf16 != 0};
}
// the two bf16 values of one 32-bit word, in memory order
__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

// ---- 1. statistics -----------------------------------------------------------------------------------
// the pointers of an argument block that was read through kernarg_block_after_requests, as global pointers again
__device__ __forceinline__ void global_pointers(AcceptArgs& a) {
    a.target = global_pointer(a.target);
    a.draft = global_pointer(a.draft);
    a.token = global_pointer(a.token);
    a.parent = global_pointer(a.parent);
    a.uniforms = global_pointer(a.uniforms);
    a.con_anchor = global_pointer(a.con_anchor);
    a.path = global_pointer(a.path);
    a.n_accepted = global_pointer(a.n_accepted);
    a.final_token = global_pointer(a.final_token);
    a.final_kind = global_pointer(a.final_kind);
    a.last_node = global_pointer(a.last_node);
    a.selected_con = global_pointer(a.selected_con);
    a.status = global_pointer(a.status);
    a.stats = global_pointer(a.stats);
    a.z_tok = global_pointer(a.z_tok);
    a.chain_z = global_pointer(a.chain_z);
    a.accept_bit = global_pointer(a.accept_bit);
    a.sampled = global_pointer(a.sampled);
    a.chain_parts = global_pointer(a.chain_parts);
}

// The kernel-argument segment of accept_stats_kernel as the launch lays it out.
struct StatsKernArgs {
    const void* target;
    const void* draft;
    int64_t row_stride;
    unsigned geometry;       // T | n_mat << 8 | logits_bf16 << 10
    int V;
    int split_len;
    float temperature;
    AcceptArgs a;
};
static_assert(offsetof(StatsKernArgs, a) == 40, "kernel-argument layout of accept_stats_kernel");

template <bool kGreedy, bool kBf16>
__global__ __launch_bounds__(kStatThreads) void accept_stats_kernel(const void* target, const void* draft,
                                                                    int64_t row_stride, unsigned geometry, int V,
                                                                    int split_len, float temperature,
                                                                    AcceptArgs /* read below */) {
    const int T = (int)(geometry & 0xffu), n_mat = (int)((geometry >> 8) & 3u);
    constexpr bool is_bf16 = kBf16;
    const int split = blockIdx.x;
    const int mat = blockIdx.y / T;
    const int row = blockIdx.y % T;
    const int b = blockIdx.z;
    const Row lrow{static_cast<const unsigned char*>(mat == 0 ? target : draft) +
                       ((int64_t)b * T + row) * row_stride * (is_bf16 ? 2 : 4), is_bf16};
    const int begin = split * split_len;
    const int end = min(V, begin + split_len);
    const float it = kGreedy ? 0.f : kLog2e / temperature;

    // Vector part: 16-byte pieces (four fp32 or eight bf16 entries), a batch of them per lane requested before the
    // first is used (a range of the usual size is one or two batches, so the workgroup pays few memory round
    // trips).  The first batch goes out before anything else, from the leading arguments alone.
    constexpr int kInFlight = 8;
    const int per = is_bf16 ? 8 : 4;
    const unsigned char* first_entry = static_cast<const unsigned char*>(lrow.p) + (int64_t)begin * (is_bf16 ? 2 : 4);
    const int n_pieces = aligned16(first_entry) ? (end - begin) / per : 0;
    // (a pointer typed as global memory: the streaming loads are global loads, not flat ones)
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    typedef const u32x4 __attribute__((address_space(1)))* global_pieces;
    const global_pieces pieces = (global_pieces)(uintptr_t)first_entry;
    auto request = [&](int i0, uint4 (&raw)[kInFlight]) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            const int i = i0 + k * kStatThreads;
            const u32x4 w = pieces[i < n_pieces ? i : i0];    // (i0 < n_pieces: the caller checks)
            raw[k] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    };
    uint4 raw[kInFlight];
    const bool any_piece = (int)threadIdx.x < n_pieces;
    if (any_piece) request(threadIdx.x, raw);

    AcceptArgs a = kernarg_block_after_requests<AcceptArgs>(offsetof(StatsKernArgs, a));
    global_pointers(a);
    a.target = target;
    a.draft = draft;
    a.row_stride = row_stride;
    a.T = T;
    a.n_mat = n_mat;
    a.logits_bf16 = is_bf16 ? 1 : 0;
    a.V = V;
    a.split_len = split_len;
    a.temperature = temperature;

    // this node's share slots of the sibling-chain kernel: "not published yet"
    if (n_mat == 2 && mat == 0 && blockIdx.x == 0) {
        unsigned long long* parts = a.chain_parts + ((int64_t)b * T + row) * a.chain_slices;
        for (int i = threadIdx.x; i < a.chain_slices; i += kStatThreads) parts[i] = 3ull;
    }

    // The logit of every child's token in this (its parent's) row, picked out by the workgroup whose range holds it:
    // the walk then finds all of them in one small array instead of gathering them from the rows.  Thread c looks
    // at node c while the first batch is on its way, so that these few dependent loads run under it; a token outside
    // the row is left alone (the walk flags the sequence).
    if (!kGreedy && threadIdx.x >= 1 && (int)threadIdx.x < T) {
        const int c = threadIdx.x;
        const int tok = a.token[(int64_t)b * T + c];
        if (a.parent[(int64_t)b * T + c] == row && tok >= begin && tok < end)
            a.z_tok[((int64_t)b * n_mat + mat) * T + c] = lrow[tok];
    }

    Red r{-INFINITY, 0x7fffffff, 0.0};
    auto consume = [&](int i0, const uint4 (&w)[kInFlight]) __attribute__((always_inline)) {
        if (!is_bf16) {
            float4 x[kInFlight];
            int v0[kInFlight];
            bool live[kInFlight];
#pragma unroll
            for (int k = 0; k < kInFlight; ++k) {
                const int i = i0 + k * kStatThreads;
                live[k] = i < n_pieces;
                v0[k] = begin + 4 * i;
                x[k] = make_float4(__uint_as_float(w[k].x), __uint_as_float(w[k].y), __uint_as_float(w[k].z),
                                   __uint_as_float(w[k].w));
            }
            red_push_batch<kGreedy, kInFlight>(r, x, v0, live, it);
        } else {
            float4 x[2 * kInFlight];
            int v0[2 * kInFlight];
            bool live[2 * kInFlight];
#pragma unroll
            for (int k = 0; k < kInFlight; ++k) {
                const int i = i0 + k * kStatThreads;
                live[2 * k] = live[2 * k + 1] = i < n_pieces;
                v0[2 * k] = begin + 8 * i;
                v0[2 * k + 1] = begin + 8 * i + 4;
                x[2 * k] = make_float4(bf16_lo(w[k].x), bf16_hi(w[k].x), bf16_lo(w[k].y), bf16_hi(w[k].y));
                x[2 * k + 1] = make_float4(bf16_lo(w[k].z), bf16_hi(w[k].z), bf16_lo(w[k].w), bf16_hi(w[k].w));
            }
            red_push_batch<kGreedy, 2 * kInFlight>(r, x, v0, live, it);
        }
    };
    if (any_piece) consume(threadIdx.x, raw);
    for (int i0 = threadIdx.x + kInFlight * kStatThreads; i0 < n_pieces; i0 += kInFlight * kStatThreads) {
        request(i0, raw);
        consume(i0, raw);
    }
    for (int i = begin + per * n_pieces + threadIdx.x; i < end; i += kStatThreads) red_push<kGreedy>(r, lrow[i], i, it);

    // wave reduction: the maximum (lowest index on ties) first, then one rescale per lane and a plain sum
    float wm = r.m;
    int wam = r.am;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float om = __shfl_xor(wm, o, kWave);
        const int oam = __shfl_xor(wam, o, kWave);
        if (om > wm || (om == wm && oam < wam)) { wm = om; wam = oam; }
    }
    double ws = 0.0;
    if (!kGreedy) {
        double s = r.s;
        if (s != 0.0 && r.m != wm) s *= rescale_factor(r.m, wm, it);
        ws = wave_sum(s);
    }
    constexpr int kStatWaves = kStatThreads / kWave;
    __shared__ float wred_m[kStatWaves];
    __shared__ int wred_am[kStatWaves];
    __shared__ double wred_s[kStatWaves];
    if ((threadIdx.x & (kWave - 1)) == 0) {
        wred_m[threadIdx.x / kWave] = wm;
        wred_am[threadIdx.x / kWave] = wam;
        wred_s[threadIdx.x / kWave] = ws;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // the waves' results: the maximum (lowest index on ties) first, then every wave's sum carried over to it
        float m = wred_m[0];
        int am = wred_am[0];
#pragma unroll
        for (int w = 1; w < kStatWaves; ++w)
            if (wred_m[w] > m || (wred_m[w] == m && wred_am[w] < am)) { m = wred_m[w]; am = wred_am[w]; }
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < kStatWaves; ++w) {
            const double sw = wred_s[w];
            sum += (sw == 0.0 || wred_m[w] == m) ? sw : sw * rescale_factor(wred_m[w], m, it);
        }
        RowStat* out = a.stats + ((((int64_t)b * a.n_mat + mat) * a.T + row) * a.splits + split);
        out->max_logit = m;
        out->argmax = (am == 0x7fffffff) ? begin : am;      // nothing above -infinity: the range's first entry
        out->sum_exp = sum;
    }
}

// Statistics of one row merged from its ranges by a group of g consecutive lanes of one wave (g a power
// of two, groups aligned to g; `sub` is the lane's index in its group).  Every lane of the wave calls
// this; lanes whose group has no row pass active = false.  All lanes of a group return the result.
constexpr int kStatBatch = 8;
// the first batch of a lane's ranges of one row (ranges sub, sub + g, ...), requested and not looked at
__device__ __forceinline__ void row_stat_request(const AcceptArgs& a, int b, int mat, int row, bool active, int sub,
                                                 int g, uint4 (&raw)[kStatBatch]) {
    const RowStat* st = a.stats + ((((int64_t)b * a.n_mat + mat) * a.T + (active ? row : 0)) * a.splits);
#pragma unroll
    for (int k = 0; k < kStatBatch; ++k) {
        const int s = sub + k * g;
        raw[k] = *reinterpret_cast<const uint4*>(st + ((active && s < a.splits) ? s : 0));
    }
}
template <bool kRequested>
__device__ __forceinline__ Red group_row_stat_impl(const AcceptArgs& a, int b, int mat, int row, bool active,
                                                   int sub, int g, float it, bool want_sum, uint4* keep,
                                                   const uint4 (&first)[kStatBatch]) {
    const RowStat* st = a.stats + ((((int64_t)b * a.n_mat + mat) * a.T + (active ? row : 0)) * a.splits);
    // A lane's ranges are sub, sub + g, ...  They are fetched kStatBatch at a time, 16 bytes each, all requested
    // before the first is looked at (a loop of single loads would pay one memory round trip per range); the
    // caller may have requested the first batch already (row_stat_request).
    auto fetch = [&](int s0, RowStat (&x)[kStatBatch], bool pre) {
#pragma unroll
        for (int k = 0; k < kStatBatch; ++k) {
            const int s = s0 + k * g;
            const uint4 w = pre ? first[k] : *reinterpret_cast<const uint4*>(st + ((active && s < a.splits) ? s : 0));
            const bool live = active && s < a.splits;     // (an entry that is not there: never the max, no mass)
            if (keep && live) keep[s] = w;                // (the caller's copy of the row's ranges, in LDS)
            x[k].max_logit = live ? __uint_as_float(w.x) : -INFINITY;
            x[k].argmax = live ? (int)w.y : 0x7fffffff;
            x[k].sum_exp = live ? __longlong_as_double((long long)(((unsigned long long)w.w << 32) | w.z)) : 0.0;
        }
    };
    RowStat head[kStatBatch];            // the lane's first batch stays in registers for the second pass
    fetch(sub, head, kRequested);
    float m = -INFINITY;
    int am = 0x7fffffff;
    auto take_max = [&](const RowStat (&x)[kStatBatch]) {
#pragma unroll
        for (int k = 0; k < kStatBatch; ++k)
            if (x[k].max_logit > m || (x[k].max_logit == m && x[k].argmax < am)) {
                m = x[k].max_logit;
                am = x[k].argmax;
            }
    };
    take_max(head);
    for (int s0 = sub + kStatBatch * g; s0 < a.splits; s0 += kStatBatch * g) {
        RowStat x[kStatBatch];
        fetch(s0, x, false);
        take_max(x);
    }
    for (int o = 1; o < g; o <<= 1) {
        const float om = __shfl_xor(m, o, kWave);
        const int oam = __shfl_xor(am, o, kWave);
        if (om > m || (om == m && oam < am)) { m = om; am = oam; }
    }
    double sum = 0.0;
    if (want_sum) {
        auto add = [&](const RowStat (&x)[kStatBatch]) {
#pragma unroll
            for (int k = 0; k < kStatBatch; ++k)
                sum += (x[k].max_logit == m) ? x[k].sum_exp : x[k].sum_exp * unnorm_prob(x[k].max_logit, m, it);
        };
        add(head);
        for (int s0 = sub + kStatBatch * g; s0 < a.splits; s0 += kStatBatch * g) {
            RowStat x[kStatBatch];
            fetch(s0, x, false);
            add(x);
        }
        for (int o = 1; o < g; o <<= 1) sum += __shfl_xor(sum, o, kWave);
    }
    return Red{m, am, sum};
}
__device__ __forceinline__ Red group_row_stat(const AcceptArgs& a, int b, int mat, int row, bool active,
                                              int sub, int g, float it, bool want_sum, uint4* keep = nullptr) {
    const uint4 none[kStatBatch] = {};
    return group_row_stat_impl<false>(a, b, mat, row, active, sub, g, it, want_sum, keep, none);
}

// ---- the law at a node after a number of rejections, one vocabulary entry at a time -------------------
struct ChainStep {        // what rejecting one child did to the laws
    int tok;              // the rejected token
    double inv_z;         // 1 / normaliser of max(p - q, 0)   (0 when the residual had no mass: p kept)
    double inv_qs;        // draft rule without replacement: 1 / (mass of q left after removing tok); else 1
    double inv_ps;        // deterministic rule: 1 / (mass of p left after removing tok)
};

template <int kRule>
__device__ __forceinline__ void law_step(int v, const ChainStep& st, double& p, double& q) {
    if (kRule == TV_RULE_DETERMINISTIC) {
        p = (v == st.tok) ? 0.0 : ((st.inv_ps > 0.0) ? p * st.inv_ps : p);
    } else {
        const double r = fmax(p - q, 0.0);
        if (st.inv_z > 0.0) p = r * st.inv_z;
        if (kRule == TV_RULE_DRAFT_WOR) q = (v == st.tok) ? 0.0 : ((st.inv_qs > 0.0) ? q * st.inv_qs : q);
    }
}

template <int kRule>
__device__ __forceinline__ void law_after(int v, double p0, double q0, const ChainStep* steps, int n,
                                          double* p_out, double* q_out) {
    double p = p0, q = q0;
    for (int i = 0; i < n; ++i) law_step<kRule>(v, steps[i], p, q);
    *p_out = p;
    *q_out = q;
}

// x of lane `src`, src the same in every lane (a register read, no LDS crossbar trip)
__device__ __forceinline__ int lane_value(int x, int src) {
    return __builtin_amdgcn_readlane(x, __builtin_amdgcn_readfirstlane(src));
}
__device__ __forceinline__ double lane_value(double x, int src) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    const int s = __builtin_amdgcn_readfirstlane(src);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, s);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), s);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

template <int kWaves>
__device__ __forceinline__ double block_sum(double x, double* scratch /* kWaves doubles */) {
    x = wave_sum(x);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[threadIdx.x / kWave] = x;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) t += scratch[w];
    return t;
}

// ---- 2. sibling chains (draft rules) --------------------------------------------------------------------
// The launch holds a whole number of groups of chain_slices workgroups.  A group takes the nodes that have
// children one after the other; each workgroup holds its slice of the node's two laws in registers and the
// group steps through the children in order.  One child costs one group-wide reduction (the normaliser of the
// corrected law): every workgroup publishes its slice's share - which stays in the workspace for the final draw -
// and collects the shares of the whole group.
//
// Forward progress does not hang on the other workgroups being resident: a workgroup polls a bounded number of
// times (wait_limit); when that runs out it computes the missing shares itself, from the rows in memory, with
// the same instruction sequence and summation order the owning workgroup uses - the same bits - and goes on.
constexpr int kChainPer = 16;                                  // vocabulary entries per lane
constexpr int kChainQuads = kChainPer / 4;
constexpr int kChainSlice = kChainThreads * kChainPer;         // vocabulary entries per workgroup

// What workgroups hand to each other inside a kernel goes through agent-scope atomic stores and loads, which
// pass by the caches that are not coherent across the device (a device-wide release fence would write back
// the whole L2); every published value carries its own "ready" tag in its two lowest mantissa bits (0 = ready,
// 3 = not yet, left there by the statistics kernel), so no second store has to be ordered behind it.  Readers
// use the value with those two bits cleared, everywhere.
__device__ __forceinline__ unsigned long long share_bits(double x) {
    return (unsigned long long)__double_as_longlong(x) & ~3ull;
}
__device__ __forceinline__ double share_value(unsigned long long bits) {
    return __longlong_as_double((long long)(bits & ~3ull));
}

// Four consecutive logits of a row (entries past the end of the row read as -infinity, which the
// laws map to zero mass).
__device__ __forceinline__ void load_quad(const Row& row, bool vec_ok, int v, int V, float* dst) {
    if (vec_ok && v + 3 < V) {
        if (row.bf16) {
            const uint2 x = *reinterpret_cast<const uint2*>(static_cast<const unsigned short*>(row.p) + v);
            dst[0] = bf16_lo(x.x); dst[1] = bf16_hi(x.x); dst[2] = bf16_lo(x.y); dst[3] = bf16_hi(x.y);
        } else {
            const float4 x = *reinterpret_cast<const float4*>(static_cast<const float*>(row.p) + v);
            dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[e] = (v + e < V) ? row[v + e] : -INFINITY;
    }
}

// This lane's kChainPer entries of the two laws at a node, for vocabulary slice `slice`: quad qd covers
// v = slice * kChainSlice + (qd * threads + tid) * 4 ...
__device__ __forceinline__ void chain_load_slice(const Row& prow, const Row& qrow, bool vec_ok, int slice, int V,
                                                 const Red& sp, const Red& sq, float it, double (&p)[kChainPer],
                                                 double (&q)[kChainPer]) {
    const double inv_sp = inv_mass(sp.s), inv_sq = inv_mass(sq.s);
    const int slice_base = slice * kChainSlice;
#pragma unroll
    for (int qd = 0; qd < kChainQuads; ++qd) {
        const int v = slice_base + (qd * kChainThreads + (int)threadIdx.x) * 4;
        float zp[4], zq[4];
        if (v < V) {
            load_quad(prow, vec_ok, v, V, zp);
            load_quad(qrow, vec_ok, v, V, zq);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) { zp[e] = -INFINITY; zq[e] = -INFINITY; }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            p[4 * qd + e] = unnorm_prob(zp[e], sp.m, it) * inv_sp;
            q[4 * qd + e] = unnorm_prob(zq[e], sq.m, it) * inv_sq;
        }
    }
}
template <int kRule>
__device__ __forceinline__ void chain_step_slice(int slice, const ChainStep& st, double (&p)[kChainPer], double (&q)[kChainPer]) {
    const int slice_base = slice * kChainSlice;
#pragma unroll
    for (int qd = 0; qd < kChainQuads; ++qd) {
        const int v = slice_base + (qd * kChainThreads + (int)threadIdx.x) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) law_step<kRule>(v + e, st, p[4 * qd + e], q[4 * qd + e]);
    }
}
// the slice's share of the normaliser of max(p - q, 0): lanes in entry order, then the workgroup's fixed tree
__device__ __forceinline__ double chain_share(const double (&p)[kChainPer], const double (&q)[kChainPer], double* red) {
    double part = 0.0;
#pragma unroll
    for (int e = 0; e < kChainPer; ++e) part += fmax(p[e] - q[e], 0.0);
    return block_sum<kChainWaves>(part, red);
}

// Every share of the j-th reduction at a node that is still missing in `shares` (tag bits set), rebuilt entry by
// entry as its owner forms it - the slice's laws from the rows, the j steps so far, the same sums in the same order,
// hence the same bits - one quad of entries at a time, so that this rarely taken path needs few registers next to
// the caller's own slice.  Called by all threads of the workgroup.
template <int kRule>
__device__ __forceinline__ void rebuild_missing_shares(const Row& prow, const Row& qrow, bool vec_ok, int V, int S,
                                                       const Red& sp, const Red& sq, float it, const ChainStep* steps,
                                                       int j, unsigned long long* shares, double* red) {
    const double inv_sp = inv_mass(sp.s), inv_sq = inv_mass(sq.s);
    for (int s = 0; s < S; ++s) {
        if ((shares[s] & 3ull) == 0ull) continue;             // (uniform: read after a barrier)
        double part = 0.0;
#pragma unroll 1
        for (int qd = 0; qd < kChainQuads; ++qd) {
            const int v = s * kChainSlice + (qd * kChainThreads + (int)threadIdx.x) * 4;
            float zp[4], zq[4];
            if (v < V) {
                load_quad(prow, vec_ok, v, V, zp);
                load_quad(qrow, vec_ok, v, V, zq);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) { zp[e] = -INFINITY; zq[e] = -INFINITY; }
            }
            double p[4], q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p[e] = unnorm_prob(zp[e], sp.m, it) * inv_sp;
                q[e] = unnorm_prob(zq[e], sq.m, it) * inv_sq;
            }
            for (int i = 0; i < j; ++i) {
                const ChainStep st = steps[i];
#pragma unroll
                for (int e = 0; e < 4; ++e) law_step<kRule>(v + e, st, p[e], q[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) part += fmax(p[e] - q[e], 0.0);
        }
        const double theirs = block_sum<kChainWaves>(part, red);
        __syncthreads();
        if (threadIdx.x == 0) shares[s] = share_bits(theirs);
    }
    __syncthreads();
}

template <int kRule>
__global__ __launch_bounds__(kChainThreads) void accept_chain_kernel(AcceptArgs a) {
    const int T = a.T, V = a.V, S = a.chain_slices;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    __shared__ int s_parent[kMaxRows];
    __shared__ int s_token[kMaxRows];
    __shared__ int s_child[kMaxRows];
    __shared__ ChainStep s_steps[kMaxRows];
    __shared__ double s_red[kChainWaves];
    __shared__ Red s_stat[2];
    __shared__ int s_internal[kMaxRows];
    __shared__ int s_has[kMaxRows];
    __shared__ int s_flag, s_k, s_missing, s_nint;
    __shared__ float s_zp[kMaxRows], s_zq[kMaxRows], s_u[kMaxRows];      // per child: its token's logits, its uniform
    extern __shared__ unsigned long long s_share[];                        // [S]: the shares of one reduction
    const int n_groups = gridDim.x / S;
    const int group = blockIdx.x / S, slice = blockIdx.x % S;
    if (group >= n_groups) return;
    int loaded_b = -1;
    for (int item = group;; item += n_groups) {
        const int b = item / T, r = item % T;
        if (b >= a.B) break;
        __syncthreads();
        if (b != loaded_b) {
            loaded_b = b;
            for (int i = tid; i < T; i += kChainThreads) {
                s_parent[i] = a.parent[(int64_t)b * T + i];
                s_token[i] = a.token[(int64_t)b * T + i];
                s_has[i] = 0;
            }
            __syncthreads();
            int bad = validate_tree(s_parent, nullptr, T, &s_flag);
            int tok_bad = 0;
            for (int i = tid; i < T; i += kChainThreads)
                if (s_token[i] < 0 || s_token[i] >= V) tok_bad = 1;
            if (tok_bad) atomicOr(&s_flag, TV_STATUS_BAD_TOKEN);
            __syncthreads();
            bad = s_flag;
            if (!bad)
                for (int i = 1 + tid; i < T; i += kChainThreads) atomicAdd(&s_has[s_parent[i]], 1);
            __syncthreads();
            if (wave == 0) {
                // The nodes that have children, those with the most children first (ties by index): a child costs
                // a round trip through the whole group, so the long chains are what the groups' loads are
                // balanced by (see the order in which a group takes its nodes, below).
                const int k_lo = (lane < T) ? s_has[lane] : 0;
                const int k_hi = (lane + kWave < T) ? s_has[lane + kWave] : 0;
                int k_max = max(k_lo, k_hi);
                for (int off = kWave / 2; off; off >>= 1) k_max = max(k_max, __shfl_xor(k_max, off));
                int n = 0;
                for (int kk = k_max; kk >= 1; --kk) {
                    unsigned long long lo = __ballot(k_lo == kk), hi = __ballot(k_hi == kk);
                    if (lo == 0 && hi == 0) continue;
                    if (lane == 0) {
                        while (lo) { s_internal[n++] = __ffsll((long long)lo) - 1; lo &= lo - 1; }
                        while (hi) { s_internal[n++] = kWave + __ffsll((long long)hi) - 1; hi &= hi - 1; }
                    }
                }
                if (lane == 0) s_nint = bad ? 0 : n;       // malformed input: nothing to do (the walk kernel reports it)
            }
            __syncthreads();
        }
        // Pass p of the groups over the sorted nodes runs forwards for even p and backwards for odd p, so the group
        // that took the longest chain of one pass takes the shortest of the next.
        // (a permutation of 0 .. T-1: the last pass may be a short one)
        const int pass = r / n_groups, pos = r % n_groups;
        const int pass_len = min(n_groups, T - pass * n_groups);
        const int ri = pass * n_groups + ((pass & 1) ? pass_len - 1 - pos : pos);
        if (ri >= s_nint) continue;
        const int u = s_internal[ri];
        if (wave == 0) {            // the children of u, in index order
            const int par_lo = (lane < T) ? s_parent[lane] : -2;
            const int par_hi = (lane + kWave < T) ? s_parent[lane + kWave] : -2;
            unsigned long long kids_lo = __ballot(par_lo == u), kids_hi = __ballot(par_hi == u);
            if (lane == 0) {
                int k = 0;
                while (kids_lo) { s_child[k++] = __ffsll((long long)kids_lo) - 1; kids_lo &= kids_lo - 1; }
                while (kids_hi) { s_child[k++] = kWave + __ffsll((long long)kids_hi) - 1; kids_hi &= kids_hi - 1; }
                s_k = k;
            }
        }
        __syncthreads();
        const int k = s_k;

        const float it = kLog2e / a.temperature;
        if (wave < 2) {         // wave 0: the target row's statistics, wave 1: the draft row's
            const Red r = group_row_stat(a, b, wave, u, true, lane, kWave, it, true);
            if (lane == 0) s_stat[wave] = r;
        }
        if (tid < k) {          // what the statistics kernel picked out of the two rows for this child
            const int c = s_child[tid];
            s_zp[tid] = a.z_tok[((int64_t)b * 2 + 0) * T + c];
            s_zq[tid] = a.z_tok[((int64_t)b * 2 + 1) * T + c];
            s_u[tid] = a.uniforms[(int64_t)b * 2 * T + c];
        }
        __syncthreads();
        const Red sp = s_stat[0], sq = s_stat[1];
        const double inv_sp = inv_mass(sp.s), inv_sq = inv_mass(sq.s);
        const Row prow = logits_row(a, a.target, b, u), qrow = logits_row(a, a.draft, b, u);
        const bool vec_ok = prow.quad_aligned() && qrow.quad_aligned();

        double p[kChainPer], q[kChainPer];
        chain_load_slice(prow, qrow, vec_ok, slice, V, sp, sq, it, p, q);

        for (int j = 0; j < k; ++j) {
            const int c = s_child[j];
            if (tid == 0) {
                // the accept test of child j, as if its earlier siblings were all rejected
                const int x = s_token[c];
                double px, qx;
                law_after<kRule>(x, unnorm_prob(s_zp[j], sp.m, it) * inv_sp, unnorm_prob(s_zq[j], sq.m, it) * inv_sq,
                                 s_steps, j, &px, &qx);
                if (slice == 0) a.accept_bit[(int64_t)b * T + c] = ((double)s_u[j] * qx < px) ? 1 : 0;
                ChainStep st;
                st.tok = x;
                st.inv_z = 0.0;
                st.inv_ps = 1.0;
                const double qs = 1.0 - qx;      // mass of q left once x is removed
                st.inv_qs = (kRule == TV_RULE_DRAFT_WOR && qs > 0.0) ? 1.0 / qs : 0.0;
                s_steps[j] = st;
                s_missing = 0;
            }
            // normaliser of the corrected law after rejecting child j: this slice's share, published in child c's
            // slot of this slice (where it also stays for the final draw) ...
            const double mine = chain_share(p, q, s_red);
            unsigned long long* parts = a.chain_parts + ((int64_t)b * T + c) * S;
            if (tid == 0)
                __hip_atomic_store(parts + slice, share_bits(mine), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // ... and the others': a bounded number of looks at every slot
            if (wave == 0) {
                int missing = 0;
                unsigned polls = 0;
                for (int s = lane; s < S; s += kWave) {
                    unsigned long long bits = share_bits(mine);
                    if (s != slice) {
                        for (;;) {
                            bits = __hip_atomic_load(parts + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            if ((bits & 3ull) == 0ull) break;
                            if (++polls > a.wait_limit) { bits = 3ull; break; }
                            __builtin_amdgcn_s_sleep(1);
                        }
                    }
                    s_share[s] = bits;
                    if ((bits & 3ull) != 0ull) missing = 1;
                }
                if (__any(missing) && lane == 0) s_missing = 1;
            }
            __syncthreads();
            if (s_missing) {
                // Some workgroup of the group has not been heard from (it may not even be running yet): its share
                // is rebuilt here (a call, so that this rarely taken path costs the loop above no registers).
                rebuild_missing_shares<kRule>(prow, qrow, vec_ok, V, S, sp, sq, it, s_steps, j, s_share, s_red);
            }
            // the whole: every workgroup of the group adds the shares in the same order
            if (wave == 0) {
                double z = 0.0;
                for (int s = lane; s < S; s += kWave) z += share_value(s_share[s]);
                z = wave_sum(z);
                if (lane == 0) {
                    s_steps[j].inv_z = (z > 0.0) ? 1.0 / z : 0.0;
                    if (slice == 0) a.chain_z[(int64_t)b * T + c] = z;
                }
            }
            __syncthreads();
            if (j + 1 < k) chain_step_slice<kRule>(slice, s_steps[j], p, q);
        }
    }   // next node of this group
}

// ---- 2b. the inverse-CDF draw from a law whose mass per piece of the vocabulary is known -------------------------
constexpr int kDrawQuads = 2;     // quads of entries a lane holds: a piece has at most 8192 entries
constexpr int kMaxPieces = 256;   // pieces a draw can choose among (four per lane of one wave)
constexpr int kKeptRanges = 2048; // reduced ranges of the target rows a walk workgroup keeps in LDS (32 KB)

struct WalkShared {
    int parent[kMaxRows];
    int token[kMaxRows];
    int path[kMaxRows];
    float unif[2 * kMaxRows];
    float m_p[kMaxRows];
    float m_q[kMaxRows];
    double inv_s_p[kMaxRows];
    double inv_s_q[kMaxRows];
    int argmax[kMaxRows];
    float z_tok_p[kMaxRows];      // target logit of node c's token in its parent's row
    float z_tok_q[kMaxRows];      // draft logit of the same entry
    int abit[kMaxRows];           // draft rules: the chain kernel's accept bit of node c
    double chain_z[kMaxRows];     // draft rules: normaliser of the corrected law after rejecting node c
    ChainStep steps[kMaxRows];    // the rejections at the stop node, in order
    int rej_child[kMaxRows];      // ... the child each of them turned down
    double rej_p0[kMaxRows];      // ... and the target's own probability of its token
    double p0[kMaxRows];          // deterministic rule: probability of node c's token under its parent's own law
    int con_anchor[kMaxRows];     // node of each contemplate row (the first kMaxRows of them)
    int verdict[kMaxRows];        // TV_STATUS_* bits of each node's own checks
    double red[kDrawWaves];
    double wave_tot[kDrawWaves];
    int wave_last[kDrawWaves];
    double base;                  // mass of the final law in the pieces before the chosen one
    int flag, cur, n_steps, rejected_any, len;
    int piece;
    int ranges_kept;              // the target rows' reduced ranges are in `ranges` (T * splits <= kKeptRanges)
    uint4 ranges[kKeptRanges];    // [node][range], as the statistics kernel wrote them
};

// One lane's contiguous run of vocabulary entries [v0, v0 + 4*quads) of the law at `node` after sh.n_steps
// rejections, from the logits zp / zq the lane holds (entries past the piece hold -infinity: no mass; quads <=
// kDrawQuads).  Leaves the entries' probabilities in pv, returns their sum (added in vocabulary order) and, in
// *last, the run's last entry that carries mass.
template <int kRule>
__device__ __forceinline__ double run_probs(const WalkShared& sh, const float (&zp)[kDrawQuads][4],
                                            const float (&zq)[kDrawQuads][4], int node, int v0, int quads, float it,
                                            double (&pv)[kDrawQuads * 4], int* last) {
    constexpr bool kDraft = (kRule == TV_RULE_DRAFT_WOR || kRule == TV_RULE_DRAFT_WR);
    int lst = -1;
    double run = 0.0;
    const float m_p = sh.m_p[node], m_q = kDraft ? sh.m_q[node] : 0.f;
    const double inv_s_p = sh.inv_s_p[node], inv_s_q = kDraft ? sh.inv_s_q[node] : 0.0;
    const int n = sh.n_steps;
#pragma unroll
    for (int g = 0; g < kDrawQuads; ++g) {
        const int v = v0 + 4 * g;
        double p[4], q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            p[e] = (g < quads) ? unnorm_prob(zp[g][e], m_p, it) * inv_s_p : 0.0;
            q[e] = (kDraft && g < quads) ? unnorm_prob(zq[g][e], m_q, it) * inv_s_q : 0.0;
        }
        if (g < quads)                              // (uniform: a short run costs no more than it holds)
            for (int i = 0; i < n; ++i) {           // one LDS read per rejection, four independent chains
                const ChainStep st = sh.steps[i];
#pragma unroll
                for (int e = 0; e < 4; ++e) law_step<kRule>(v + e, st, p[e], q[e]);
            }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            pv[4 * g + e] = p[e];
            run += p[e];
            if (p[e] > 0.0) lst = v + e;
        }
    }
    *last = lst;
    return run;
}

// The first v at which the running sum of the law at `node` (after sh.n_steps rejections) exceeds u, in two
// steps.  The law's mass in each of n_pieces consecutive pieces of piece_len entries comes from mass_of(piece) - no
// pass over the vocabulary - so only the piece that holds the crossing is read, by this one workgroup.
// Step 1, choose_piece: the 64 lanes of ONE wave find that piece and leave it (and the mass in front of it) in sh.
// A workgroup barrier must follow before step 2.
template <typename MassFn>
__device__ __forceinline__ void choose_piece(WalkShared& sh, double u, int n_pieces, MassFn mass_of) {
    const int lane = threadIdx.x & (kWave - 1);
    {
        // prefix sum over the pieces in vocabulary order (a lane holds kPer consecutive ones), first piece at which
        // the running sum exceeds u; if rounding leaves the total at or below u, the last piece that carries mass
        constexpr int kPer = kMaxPieces / kWave;
        const int per = (n_pieces + kWave - 1) / kWave;        // (one piece per lane up to 64 pieces: all fetched at once)
        double pm[kPer], mine = 0.0;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int s = lane * per + k;
            pm[k] = (k < per && s < n_pieces) ? mass_of(s) : 0.0;
            mine += pm[k];
        }
        const double inc = wave_prefix_sum(mine);
        double run = inc - mine, base_c = 0.0;
        int cand = -1, has_mass = -1;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            if (cand < 0 && k < per && lane * per + k < n_pieces && run + pm[k] > u) { cand = lane * per + k; base_c = run; }
            if (pm[k] > 0.0) has_mass = lane * per + k;
            run += pm[k];
        }
        const unsigned long long hit = __ballot(cand >= 0);
        int piece;
        double base = 0.0;
        if (hit) {
            const int first = __ffsll((long long)hit) - 1;
            piece = lane_value(cand, first);
            base = lane_value(base_c, first);
        } else {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) has_mass = max(has_mass, __shfl_xor(has_mass, o, kWave));
            piece = has_mass;               // (-1: no mass anywhere)
            base = -4.0;                    // no running sum inside it exceeds u: its last entry with mass is taken
        }
        if (lane == 0) {
            sh.piece = piece;
            sh.base = base;
        }
    }
}

// Step 2, draw_in_piece: every thread of the workgroup calls this (after the barrier that follows choose_piece); the
// token (-1: the law has no mass at all) is written to *out_tok by exactly one thread.
template <int kRule>
__device__ __forceinline__ void draw_in_piece(const AcceptArgs& a, WalkShared& sh, int b, int node, double u, float it,
                                              int piece_len, int32_t* out_tok) {
    constexpr bool kDraft = (kRule == TV_RULE_DRAFT_WOR || kRule == TV_RULE_DRAFT_WR);
    const int V = a.V;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int piece = sh.piece;
    if (piece < 0) {
        if (tid == 0) *out_tok = -1;
        return;
    }

    // the chosen piece, a contiguous run of quads per lane in vocabulary order
    const Row prow = logits_row(a, a.target, b, node);
    const Row qrow = kDraft ? logits_row(a, a.draft, b, node) : prow;
    const bool vec_ok = prow.quad_aligned() && qrow.quad_aligned();
    const int begin = piece * piece_len, end = min(V, begin + piece_len);
    const int quads = (end - begin + 4 * kDrawThreads - 1) / (4 * kDrawThreads);      // <= kDrawQuads (plan_accept)
    const int v0 = begin + tid * 4 * quads;
    // the lane's logits, all requested before the first is used; they stay in registers for the second pass
    float zp[kDrawQuads][4], zq[kDrawQuads][4];
#pragma unroll
    for (int g = 0; g < kDrawQuads; ++g) {
        const int v = v0 + 4 * g;
        if (g < quads && v < end) {
            load_quad(prow, vec_ok, v, end, zp[g]);       // entries past the piece read as -infinity: no mass
            if (kDraft) load_quad(qrow, vec_ok, v, end, zq[g]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) zp[g][e] = -INFINITY;
        }
        if (!kDraft || !(g < quads && v < end)) {
#pragma unroll
            for (int e = 0; e < 4; ++e) zq[g][e] = -INFINITY;
        }
    }
    int last;
    double pv[kDrawQuads * 4];
    const double mine = run_probs<kRule>(sh, zp, zq, node, v0, quads, it, pv, &last);
    // every wave's total (one LDS word per wave, no atomics)
    const double inc = wave_prefix_sum(mine);
    if (lane == kWave - 1) sh.wave_tot[wave] = inc;
    __syncthreads();
    // the wave in which the running sum crosses u (every wave finds the same one: lane w looks at wave w)
    static_assert(kDrawWaves <= kWave, "one lane per wave");
    const double w_tot = (lane < kDrawWaves) ? sh.wave_tot[lane] : 0.0;
    const double w_inc = wave_prefix_sum(w_tot);          // (lanes past the waves hold 0)
    const unsigned long long w_over = __ballot(lane < kDrawWaves && sh.base + w_inc > u);
    if (!w_over) {
        // No wave's running sum exceeds u: the piece sums put the crossing here, the in-order sums round just below
        // it, or the total itself rounds to u or less - the last entry of the piece that carries mass is taken.
        // (Rare, and the same in every wave - all of them formed w_over from the same LDS words - so the barrier
        //  below is met by the whole workgroup.)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o, kWave));
        if (lane == kWave - 1) sh.wave_last[wave] = last;
        __syncthreads();
        int piece_last = (lane < kDrawWaves) ? sh.wave_last[lane] : -1;
#pragma unroll
        for (int o = 1; o < kDrawWaves; o <<= 1) piece_last = max(piece_last, __shfl_xor(piece_last, o, kWave));
        if (tid == 0) *out_tok = lane_value(piece_last, 0);
        return;
    }
    const int w_star = __ffsll((long long)w_over) - 1;
    const double before = sh.base + lane_value(w_inc - w_tot, w_star);
    if (wave == w_star) {
        const unsigned long long over = __ballot(before + inc > u);       // not empty: the wave's total exceeds u
        const int l_star = __ffsll((long long)over) - 1;
        if (lane == l_star) {
            // this lane's run holds the crossing: its entries again, in order, from the running sum in front of them
            // (if the sums formed here round just below u, the run's last entry with mass)
            double run = before + (inc - mine);
            int fnd = -1, lst = -1;
#pragma unroll
            for (int e = 0; e < kDrawQuads * 4; ++e) {
                run += pv[e];
                if (pv[e] > 0.0) lst = v0 + e;
                if (fnd < 0 && run > u) fnd = v0 + e;
            }
            *out_tok = (fnd >= 0) ? fnd : lst;
        }
    }
}

// mass of range `s` of the target row at `node`, as a share of the row (statistics kernel's ranges)
__device__ __forceinline__ double range_mass(const AcceptArgs& a, const WalkShared& sh, int b, int node, int s, float it) {
    RowStat st;
    if (sh.ranges_kept) {
        const uint4 w = sh.ranges[node * a.splits + s];
        st.max_logit = __uint_as_float(w.x);
        st.sum_exp = __longlong_as_double((long long)(((unsigned long long)w.w << 32) | w.z));
    } else {
        st = a.stats[(((int64_t)b * a.n_mat) * a.T + node) * a.splits + s];
    }
    const float m = sh.m_p[node];
    return ((st.max_logit == m) ? st.sum_exp : st.sum_exp * unnorm_prob(st.max_logit, m, it)) * sh.inv_s_p[node];
}

// The target's own token at every node (sample-and-match rule).  Grid (T, B): one workgroup draws, for one node,
// the token that plain sampling of the target would emit there: inverse CDF of softmax(target row /
// temperature) at the node's uniform u[T + node].
__global__ __launch_bounds__(kDrawThreads) void accept_sample_kernel(AcceptArgs a) {
    const int i = blockIdx.x, b = blockIdx.y;
    __shared__ WalkShared sh;
    const float it = kLog2e / a.temperature;
    if (threadIdx.x < kWave) {
        const Red st = group_row_stat(a, b, 0, i, true, threadIdx.x, kWave, it, true);
        if (threadIdx.x == 0) {
            sh.m_p[i] = st.m;
            sh.inv_s_p[i] = inv_mass(st.s);
            sh.n_steps = 0;
            sh.ranges_kept = 0;
        }
    }
    __syncthreads();
    const double u = (double)a.uniforms[(int64_t)b * 2 * a.T + a.T + i];
    if (threadIdx.x < kWave) choose_piece(sh, u, a.splits, [&](int s) { return range_mass(a, sh, b, i, s, it); });
    __syncthreads();
    draw_in_piece<TV_RULE_SAMPLE_MATCH>(a, sh, b, i, u, it, a.split_len, a.sampled + (int64_t)b * a.T + i);
}

// ---- 3. walk + final draw ---------------------------------------------------------------------------------
// One workgroup per sequence.  What its first loads hang on comes as leading arguments of their own, which are in
// registers when a wave starts (kernel-argument preload, see the build flags): the argument block itself costs a
// memory round trip.
// The kernel-argument segment of accept_walk_kernel as the launch lays it out (arguments in order, each at its
// natural alignment).
struct WalkKernArgs {
    const RowStat* stats;
    const float* z_tok;
    const int32_t* parent;
    const int32_t* token;
    const float* uniforms;
    unsigned geometry;
    float temperature;
    AcceptArgs a;
};
static_assert(offsetof(WalkKernArgs, a) == 48, "kernel-argument layout of accept_walk_kernel");

template <int kRule>
__global__ __launch_bounds__(kDrawThreads) void accept_walk_kernel(const RowStat* stats, const float* z_tok,
                                                                   const int32_t* parent, const int32_t* token,
                                                                   const float* uniforms, unsigned geometry,
                                                                   float temperature, AcceptArgs /* read below */) {
    __shared__ WalkShared sh;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    // sample-and-match walks like greedy, with the node's sampled token in the place of the row's argmax
    constexpr bool kMatch = (kRule == TV_RULE_SAMPLE_MATCH);
    constexpr bool kGreedy = (kRule == TV_RULE_GREEDY) || kMatch;
    constexpr bool kDraft = (kRule == TV_RULE_DRAFT_WOR || kRule == TV_RULE_DRAFT_WR);
    const float it = kGreedy ? 0.f : kLog2e / temperature;

    // The reduced ranges of every row are requested first, from the leading arguments alone (they are in registers
    // when the wave starts); the argument block is read after that, so that its memory round trip runs under the
    // requests' instead of in front of them.
    AcceptArgs lead{};
    lead.stats = const_cast<RowStat*>(stats);
    lead.T = (int)(geometry & 0xffu);
    lead.splits = (int)((geometry >> 8) & 0xfffu);
    lead.n_mat = (int)(geometry >> 20);
    const int T = lead.T;
    const int n_rows = kMatch ? 0 : T * (kDraft ? 2 : 1);
    int g = 1;                                   // lanes that share one row's ranges: one batch of loads per lane,
    while ((lead.splits + g - 1) / g > 8 && g < kWave) g *= 2;                      // more lanes while there are spare ones
    while (2 * g * n_rows <= kDrawThreads && lead.splits / (2 * g) >= 3 && g < kWave) g *= 2;
    const int per_pass = kDrawThreads / g;
    uint4 first_raw[kStatBatch];
    {
        const int r = tid / g;
        const bool active = r < n_rows;
        const int mat = (active && r >= T) ? 1 : 0, i = active ? r - mat * T : 0;
        if (!kMatch) row_stat_request(lead, b, mat, i, active, tid % g, g, first_raw);
    }
    // ... and so is what the walk needs per node - the tree, the tokens, the uniforms, every child's token logit -
    // by the workgroup's last waves (thread 1023 - i takes node i; kMaxRows < kDrawThreads), into registers for now
    const int my_node = kDrawThreads - 1 - tid;
    const bool has_node = my_node < T;
    int r_parent = 0, r_token = 0;
    float r_u0 = 0.f, r_u1 = 0.f, r_zp = 0.f;
    if (has_node) {
        r_parent = parent[(int64_t)b * T + my_node];
        r_token = token[(int64_t)b * T + my_node];
        if (!kGreedy) {
            r_u0 = uniforms[(int64_t)b * 2 * T + my_node];
            r_u1 = uniforms[(int64_t)b * 2 * T + T + my_node];
            r_zp = z_tok[((int64_t)b * lead.n_mat) * T + my_node];               // (entry 0, the root's, is never read)
        }
    }
    AcceptArgs a = kernarg_block_after_requests<AcceptArgs>(offsetof(WalkKernArgs, a));
    global_pointers(a);
    a.stats = const_cast<RowStat*>(stats);
    a.z_tok = const_cast<float*>(z_tok);
    a.parent = parent;
    a.token = token;
    a.uniforms = uniforms;
    a.T = lead.T;
    a.splits = lead.splits;
    a.n_mat = lead.n_mat;
    a.temperature = temperature;
    const int V = a.V;

    // what hangs on the argument block: the draft rules' per-node results of the chain kernel, the sampled tokens,
    // the contemplate rows' anchors (needed at the very end: fetched now, with everything else).  All of these
    // loads are issued before the first value is stored, so that they share one memory round trip.
    float r_zq = 0.f;
    int r_abit = 0, r_sampled = 0;
    double r_chain_z = 0.0;
    if (has_node) {
        if (kDraft) {
            r_zq = a.z_tok[((int64_t)b * a.n_mat + 1) * T + my_node];
            r_abit = a.accept_bit[(int64_t)b * T + my_node];
            r_chain_z = a.chain_z[(int64_t)b * T + my_node];
        }
        if (kMatch) r_sampled = a.sampled[(int64_t)b * T + my_node];
    }
    constexpr int kConPer = kMaxRows / kWave;
    int r_con[kConPer];
    int n_con_here = 0;
    if (wave == kDrawWaves - 1) {
        n_con_here = (a.selected_con && a.con_anchor) ? min(a.C, kMaxRows) : 0;
#pragma unroll
        for (int j = 0; j < kConPer; ++j) {
            const int i = j * kWave + (kWave - 1 - lane);
            r_con[j] = (i < n_con_here) ? a.con_anchor[(int64_t)b * a.C + i] : -1;
        }
    }
    if (has_node) {
        // this node's checks, on the values just fetched: the verdicts are in LDS with everything else, so that the
        // one barrier below is all the checks cost (acceptance trees have exactly one root, node 0)
        int verdict = 0;
        if (r_parent < -1 || r_parent >= my_node || (my_node > 0 && r_parent < 0)) verdict |= TV_STATUS_BAD_PARENT;
        if (r_token < 0 || r_token >= V) verdict |= TV_STATUS_BAD_TOKEN;
        sh.verdict[my_node] = verdict;
        sh.parent[my_node] = r_parent;
        sh.token[my_node] = r_token;
        if (!kGreedy) {
            sh.unif[my_node] = r_u0;
            sh.unif[T + my_node] = r_u1;
            sh.z_tok_p[my_node] = r_zp;
            if (kDraft) {
                sh.z_tok_q[my_node] = r_zq;
                sh.abit[my_node] = r_abit;
                sh.chain_z[my_node] = r_chain_z;
            }
        }
        if (kMatch) sh.argmax[my_node] = r_sampled;
    }
    if (wave == kDrawWaves - 1) {
#pragma unroll
        for (int j = 0; j < kConPer; ++j) {
            const int i = j * kWave + (kWave - 1 - lane);
            if (i < n_con_here) sh.con_anchor[i] = r_con[j];
        }
    }
    const bool keep_ranges = !kGreedy && !kMatch && T * a.splits <= kKeptRanges;
    if (tid == 0) sh.ranges_kept = keep_ranges ? 1 : 0;
    if (!kMatch) {
        for (int r0 = 0; r0 < n_rows; r0 += per_pass) {
            if (r0 + (wave * kWave) / g >= n_rows) break;      // no row for this wave in this pass, nor in a later one
            const int r = r0 + tid / g;
            const bool active = r < n_rows;
            const int mat = (active && r >= T) ? 1 : 0, i = active ? r - mat * T : 0;
            uint4* keep = (keep_ranges && active && mat == 0) ? sh.ranges + i * a.splits : nullptr;
            const Red st = (r0 == 0)
                ? group_row_stat_impl<true>(a, b, mat, i, active, tid % g, g, it, !kGreedy, keep, first_raw)
                : group_row_stat_impl<false>(a, b, mat, i, active, tid % g, g, it, !kGreedy, keep, first_raw);
            if (active && tid % g == 0) {
                if (mat == 0) {
                    sh.m_p[i] = st.m;
                    sh.argmax[i] = st.am;
                    sh.inv_s_p[i] = kGreedy ? 0.0 : inv_mass(st.s);
                } else {
                    sh.m_q[i] = st.m;
                    sh.inv_s_q[i] = inv_mass(st.s);
                }
            }
        }
    }
    __syncthreads();
    // the target's own probability of every node's token at its parent, all nodes at once (two per lane): by the
    // wave that walks, which then only reads them back - no barrier in between
    if (kRule == TV_RULE_DETERMINISTIC && wave == 0) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int c = lane + k * kWave;
            if (c >= 1 && c < T) {
                const int pc = sh.parent[c];
                if (pc >= 0 && pc < c) sh.p0[c] = unnorm_prob(sh.z_tok_p[c], sh.m_p[pc], it) * sh.inv_s_p[pc];
            }
        }
    }
    // every wave gathers the nodes' verdicts for itself (two LDS reads per lane, one vote per status bit)
    int bad = 0;
    {
        static_assert(kMaxRows <= 2 * kWave, "two nodes per lane");
        const int v = ((lane < T) ? sh.verdict[lane] : 0) | ((lane + kWave < T) ? sh.verdict[lane + kWave] : 0);
        if (__ballot(v & TV_STATUS_BAD_PARENT)) bad |= TV_STATUS_BAD_PARENT;
        if (__ballot(v & TV_STATUS_BAD_TOKEN)) bad |= TV_STATUS_BAD_TOKEN;
    }
    int32_t* path = a.path + (int64_t)b * T;
    if (bad) {
        for (int i = tid; i < T; i += kDrawThreads) path[i] = -1;
        if (tid == 0) {
            a.status[b] = bad;
            a.n_accepted[b] = -1;
            a.final_token[b] = -1;
            a.final_kind[b] = -1;
            a.last_node[b] = -1;
            if (a.selected_con) a.selected_con[b] = -1;
        }
        return;
    }

    // the walk: wave 0, LDS only.  Every lane follows the same path (the tests are wave-uniform); the
    // lanes only share the search for a node's children, which a ballot over the parent array gives in
    // index order (a child's index exceeds its parent's).
    // Deterministic rule: what the rejections at the current node did is also kept in registers, lane i holding
    // rejection i (the first 64; the workgroup's copy in LDS holds all), so that replaying them for the next child
    // and, later, for the pieces of the final law costs register reads instead of one LDS round trip per step.
    int rg_tok = -1;
    double rg_inv_ps = 0.0, rg_p0 = 0.0;
    if (wave == 0) {
        const int par_lo = (lane < T) ? sh.parent[lane] : -2;
        const int par_hi = (lane + kWave < T) ? sh.parent[lane + kWave] : -2;
        int cur = 0, len = 0, nrej = 0;
        if (lane == 0) sh.path[0] = 0;
        for (;;) {
            nrej = 0;
            int next = -1;
            unsigned long long kids_lo = __ballot(par_lo == cur), kids_hi = __ballot(par_hi == cur);
            while (kids_lo | kids_hi) {
                int c;
                if (kids_lo) { c = __ffsll((long long)kids_lo) - 1; kids_lo &= kids_lo - 1; }
                else { c = kWave + __ffsll((long long)kids_hi) - 1; kids_hi &= kids_hi - 1; }
                const int x = sh.token[c];
                bool acc;
                if (kGreedy) {
                    acc = (x == sh.argmax[cur]);
                } else if (kRule == TV_RULE_DETERMINISTIC) {
                    const double p0 = sh.p0[c];
                    const float uc = sh.unif[c];             // (requested with the other two, not behind the replay)
                    asm volatile("" : : "v"(uc));
                    double p = p0;
                    for (int i = 0; i < nrej; ++i) {         // (law_step of the deterministic rule, step by step)
                        const int tk = (i < kWave) ? lane_value(rg_tok, i) : sh.steps[i].tok;
                        const double ips = (i < kWave) ? lane_value(rg_inv_ps, i) : sh.steps[i].inv_ps;
                        p = (x == tk) ? 0.0 : ((ips > 0.0) ? p * ips : p);
                    }
                    acc = ((double)uc < p);
                    if (!acc) {
                        const double ps = 1.0 - p;       // mass of p left once x is removed
                        const double ips = (ps > 0.0) ? 1.0 / ps : 0.0;
                        sh.steps[nrej] = ChainStep{x, 0.0, 0.0, ips};
                        sh.rej_child[nrej] = c;
                        sh.rej_p0[nrej] = p0;
                        if (lane == nrej) { rg_tok = x; rg_inv_ps = ips; rg_p0 = p0; }
                    }
                } else {
                    acc = (sh.abit[c] != 0);
                    if (!acc) {
                        // rebuild the chain step exactly as the chain kernel formed it
                        double p, q;
                        law_after<kRule>(x, unnorm_prob(sh.z_tok_p[c], sh.m_p[cur], it) * sh.inv_s_p[cur],
                                         unnorm_prob(sh.z_tok_q[c], sh.m_q[cur], it) * sh.inv_s_q[cur],
                                         sh.steps, nrej, &p, &q);
                        const double z = sh.chain_z[c];
                        const double qs = 1.0 - q;
                        sh.steps[nrej] = ChainStep{x, (z > 0.0) ? 1.0 / z : 0.0,
                                                   (kRule == TV_RULE_DRAFT_WOR && qs > 0.0) ? 1.0 / qs : 0.0, 1.0};
                        sh.rej_child[nrej] = c;
                    }
                }
                if (acc) { next = c; break; }
                ++nrej;
            }
            if (next < 0) break;
            cur = next;
            sh.path[++len] = cur;
        }
        for (int i = len + 1 + lane; i < T; i += kWave) sh.path[i] = -1;
        sh.cur = cur;                    // (every lane stores the same values)
        sh.len = len;
        sh.n_steps = nrej;
        sh.rejected_any = (nrej > 0);
        if (!kGreedy) {
            // ---- inverse CDF at the stop node, first step: the piece of the vocabulary that holds the crossing, found
            //      by this wave right behind its walk (the other waves are still at the barrier below)
            const double u = (double)sh.unif[T + cur];
            const int n = nrej;
            // the last rejection that changed the target's law (draft rules: one whose corrected law had mass)
            int eff = -1;
            if (kDraft)
                for (int i = 0; i < n; ++i)
                    if (sh.steps[i].inv_z > 0.0) eff = i;
            if (kDraft && eff >= 0) {
                // the corrected law after that rejection: its mass per slice of the sibling-chain kernel is that
                // kernel's share of the normaliser, over the normaliser
                const unsigned long long* parts = a.chain_parts + ((int64_t)b * T + sh.rej_child[eff]) * a.chain_slices;
                const double inv_z = sh.steps[eff].inv_z;
                choose_piece(sh, u, a.chain_slices, [&](int s) { return share_value(parts[s]) * inv_z; });
            } else {
                // the target's own law with the rejected tokens taken out (deterministic rule), scaled up accordingly:
                // per range of the statistics kernel, the range's share minus the rejected tokens that lie in it
                // (this wave's lanes hold the rejections; more than 64 of them: from LDS)
                const bool in_regs = (kRule == TV_RULE_DETERMINISTIC) && n <= kWave;
                double scale = 1.0;
                int rg_first = 1;                // rejection `lane` is the first one of its token (a token proposed twice)
                if (kRule == TV_RULE_DETERMINISTIC) {
                    if (in_regs) {
                        for (int i = 0; i < n; ++i) {
                            const double ips = lane_value(rg_inv_ps, i);
                            if (ips > 0.0) scale *= ips;
                            if (lane > i && rg_tok == lane_value(rg_tok, i)) rg_first = 0;
                        }
                    } else {
                        for (int i = 0; i < n; ++i)
                            if (sh.steps[i].inv_ps > 0.0) scale *= sh.steps[i].inv_ps;
                    }
                }
                choose_piece(sh, u, a.splits, [&](int s) {
                    double m = range_mass(a, sh, b, cur, s, it);
                    if (kRule == TV_RULE_DETERMINISTIC) {
                        const int lo = s * a.split_len, hi = lo + a.split_len;
                        if (in_regs) {
                            for (int i = 0; i < n; ++i) {
                                const int x = lane_value(rg_tok, i);
                                const int first = lane_value(rg_first, i);
                                const double p0 = lane_value(rg_p0, i);
                                if (first && x >= lo && x < hi) m -= p0;
                            }
                        } else {
                            for (int i = 0; i < n; ++i) {
                                const int x = sh.steps[i].tok;
                                bool first = (x >= lo && x < hi);
                                for (int k = 0; k < i; ++k) first = first && (sh.steps[k].tok != x);     // (a token proposed twice)
                                if (first) m -= sh.rej_p0[i];
                            }
                        }
                        m = fmax(m, 0.0) * scale;
                    }
                    return m;
                });
            }
        }
    }
    __syncthreads();
    const int cur = sh.cur;

    if (kGreedy) {
        if (tid == 0) a.final_token[b] = sh.argmax[cur];
    } else {
        // ---- second step: the chosen piece is read, by the whole workgroup; the thread that finds the crossing writes
        //      the token
        const double u = (double)sh.unif[T + cur];
        const int n = sh.n_steps;
        bool corrected = false;          // (draft rules: the final law is a corrected one, cut into the chain kernel's slices)
        if (kDraft)
            for (int i = 0; i < n; ++i)
                if (sh.steps[i].inv_z > 0.0) corrected = true;
        draw_in_piece<kRule>(a, sh, b, cur, u, it, corrected ? kChainSlice : a.split_len, a.final_token + b);
    }
    for (int i = tid; i < T; i += kDrawThreads) path[i] = sh.path[i];
    if (tid == 0) {
        a.status[b] = TV_STATUS_OK;
        a.n_accepted[b] = sh.len;
        a.final_kind[b] = sh.rejected_any ? TV_FINAL_RESIDUAL : TV_FINAL_BONUS;
        a.last_node[b] = cur;
        if (a.selected_con) {
            const int n_con = a.con_anchor ? min(a.C, kMaxRows) : 0;
            int sel = -1;
            for (int c = 0; c < n_con && sel < 0; ++c)
                if (sh.con_anchor[c] == cur) sel = c;
            if (a.con_anchor)                                    // (more rows than the table holds: the rest from memory)
                for (int c = n_con; c < a.C && sel < 0; ++c)
                    if (a.con_anchor[(int64_t)b * a.C + c] == cur) sel = c;
            a.selected_con[b] = sel;
        }
    }
}

}  // namespace

int plan_accept(const tv_accept_desc& d, AcceptPlan* plan) {
    AcceptPlan p{};
    p.n_mat = (d.rule == TV_RULE_DRAFT_WOR || d.rule == TV_RULE_DRAFT_WR) ? 2 : 1;
    // about a thousand workgroups (four per CU), ranges no shorter than 4096 entries and - so that a workgroup can
    // hold one in registers when it looks for the crossing of a draw - no longer than 8192 where 64 ranges suffice
    const int rows = d.B * d.T * p.n_mat;
    int splits = (1024 + rows - 1) / rows;
    const int max_splits = (d.V + 4095) / 4096;
    const int min_splits = (d.V + kDrawQuads * 4 * kDrawThreads - 1) / (kDrawQuads * 4 * kDrawThreads);
    if (splits > max_splits) splits = max_splits;
    if (splits < min_splits) splits = min_splits;
    if (splits < 1) splits = 1;
    if (splits > kMaxPieces) splits = kMaxPieces;
    int len = (d.V + splits - 1) / splits;
    len = (len + 7) / 8 * 8;          // ranges start on a 16-byte boundary of an aligned row (fp32 and bf16)
    p.splits = (d.V + len - 1) / len;
    p.split_len = len;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    p.stats_bytes = up((size_t)rows * p.splits * sizeof(RowStat));
    p.ztok_bytes = up((size_t)rows * sizeof(float));
    p.chain_bytes = up((size_t)d.B * d.T * sizeof(double));
    p.bits_bytes = up((size_t)d.B * d.T * sizeof(int32_t));
    // the sibling chains: one group of workgroups per node, one slice of kChainSlice entries each; every child
    // keeps the shares of its reduction
    p.chain_slices = (d.V + kChainSlice - 1) / kChainSlice;
    if (p.n_mat == 2 && p.chain_slices > kMaxPieces) return TV_ERR_UNSUPPORTED;
    if (p.split_len > kDrawQuads * 4 * kDrawThreads) return TV_ERR_UNSUPPORTED;      // (a vocabulary beyond two million entries)
    p.chain_parts_bytes = (p.n_mat == 2) ? up((size_t)d.B * d.T * p.chain_slices * sizeof(double)) : 0;
    p.total_bytes = p.stats_bytes + p.ztok_bytes + p.chain_bytes + p.bits_bytes + p.chain_parts_bytes;
    *plan = p;
    return TV_OK;
}

// Workgroups of the chain kernel that fit on the current device at once (0 if unknown): the launch is sized to
// that, so that the groups' workgroups usually meet each other running (nothing breaks when they do not).
static int chain_resident_workgroups(int rule, size_t dyn_smem) {
    static std::atomic<int> cache[2][64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    std::atomic<int>& c = cache[rule == TV_RULE_DRAFT_WOR ? 0 : 1][dev];
    int v = c.load(std::memory_order_relaxed);
    if (v == 0) {
        int per_cu = 0, cus = 0;
        const hipError_t e1 = (rule == TV_RULE_DRAFT_WOR)
            ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, accept_chain_kernel<TV_RULE_DRAFT_WOR>, kChainThreads, dyn_smem)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, accept_chain_kernel<TV_RULE_DRAFT_WR>, kChainThreads, dyn_smem);
        const hipError_t e2 = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e1 == hipSuccess && e2 == hipSuccess && per_cu > 0 && cus > 0) v = per_cu * cus;
        c.store(v, std::memory_order_relaxed);
    }
    return v;
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t s) {
    const dim3 gs(a.splits, a.T * a.n_mat, a.B);
    static_assert(kMaxRows <= 0xff, "packed geometry argument of the statistics kernel");
    const unsigned stat_geometry = (unsigned)a.T | ((unsigned)a.n_mat << 8) | ((a.logits_bf16 ? 1u : 0u) << 10);
#define TV_LAUNCH_STATS(G, H) \
    accept_stats_kernel<G, H><<<gs, kStatThreads, 0, s>>>(a.target, a.draft, a.row_stride, stat_geometry, a.V, a.split_len, \
                                                          a.temperature, a)
    if (a.rule == TV_RULE_GREEDY) { if (a.logits_bf16) TV_LAUNCH_STATS(true, true); else TV_LAUNCH_STATS(true, false); }
    else { if (a.logits_bf16) TV_LAUNCH_STATS(false, true); else TV_LAUNCH_STATS(false, false); }
#undef TV_LAUNCH_STATS
    if (a.rule == TV_RULE_DRAFT_WOR || a.rule == TV_RULE_DRAFT_WR) {
        // whole groups only; as many as the device holds at once (fewer when that is unknown: one group)
        const size_t dyn = (size_t)a.chain_slices * sizeof(unsigned long long);
        const int cap = chain_resident_workgroups(a.rule, dyn);
        int groups = cap / a.chain_slices;
        if (groups < 1) groups = 1;
        if (groups > a.B * a.T) groups = a.B * a.T;
        const unsigned gc = (unsigned)groups * (unsigned)a.chain_slices;
        if (a.rule == TV_RULE_DRAFT_WOR) accept_chain_kernel<TV_RULE_DRAFT_WOR><<<gc, kChainThreads, dyn, s>>>(a);
        else accept_chain_kernel<TV_RULE_DRAFT_WR><<<gc, kChainThreads, dyn, s>>>(a);
    }
    if (a.rule == TV_RULE_SAMPLE_MATCH) accept_sample_kernel<<<dim3(a.T, a.B), kDrawThreads, 0, s>>>(a);
    const dim3 gw((unsigned)a.B);
    static_assert(kMaxRows <= 0xff && kMaxPieces <= 0xfff && kMaxRows < kDrawThreads && kMaxRows % kWave == 0,
                  "packed geometry argument of the walk kernel; one thread per node");
    const unsigned geometry = (unsigned)a.T | ((unsigned)a.splits << 8) | ((unsigned)a.n_mat << 20);
    switch (a.rule) {
        case TV_RULE_GREEDY: accept_walk_kernel<TV_RULE_GREEDY><<<gw, kDrawThreads, 0, s>>>(a.stats, a.z_tok, a.parent, a.token, a.uniforms, geometry, a.temperature, a); break;
        case TV_RULE_SAMPLE_MATCH: accept_walk_kernel<TV_RULE_SAMPLE_MATCH><<<gw, kDrawThreads, 0, s>>>(a.stats, a.z_tok, a.parent, a.token, a.uniforms, geometry, a.temperature, a); break;
        case TV_RULE_DETERMINISTIC: accept_walk_kernel<TV_RULE_DETERMINISTIC><<<gw, kDrawThreads, 0, s>>>(a.stats, a.z_tok, a.parent, a.token, a.uniforms, geometry, a.temperature, a); break;
        case TV_RULE_DRAFT_WOR: accept_walk_kernel<TV_RULE_DRAFT_WOR><<<gw, kDrawThreads, 0, s>>>(a.stats, a.z_tok, a.parent, a.token, a.uniforms, geometry, a.temperature, a); break;
        default: accept_walk_kernel<TV_RULE_DRAFT_WR><<<gw, kDrawThreads, 0, s>>>(a.stats, a.z_tok, a.parent, a.token, a.uniforms, geometry, a.temperature, a); break;
    }
    return hipGetLastError();
}

}  // namespace tv
