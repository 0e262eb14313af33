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
//   2. accept_chain_kernel   draft rules only.  A node's accept test depends only on its parent's two
//                            rows and on its rank among its siblings (as if all earlier siblings were
//                            rejected), so every parent is processed independently: one workgroup per
//                            parent walks its children in order and needs one vocabulary-wide
//                            reduction (the corrected law's normaliser) per child.
//   3. accept_walk_kernel    one workgroup per sequence: follows the accept bits from the root, then
//                            draws the final token by inverse CDF at the stop node.
#include "tv_internal.hpp"

namespace tv {

namespace {

constexpr int kStatThreads = 256;
constexpr int kWalkThreads = 1024;
constexpr int kWalkWaves = kWalkThreads / kWave;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// exp((z - m) / temperature) as the kernels evaluate it everywhere: fp32 exponent, fp64 afterwards.
__device__ __forceinline__ double unnorm_prob(float z, float m, float it_log2e) {
    return (double)fast_exp2((z - m) * it_log2e);
}

struct Red {          // (max, lowest argmax, sum exp relative to max)
    float m;
    int am;
    double s;
};

__device__ __forceinline__ Red red_merge(const Red& a, const Red& b, float it_log2e) {
    Red r;
    if (a.m > b.m || (a.m == b.m && a.am <= b.am)) { r.m = a.m; r.am = a.am; }
    else { r.m = b.m; r.am = b.am; }
    // rescaling happens once per merge of already reduced values: use the fp64 exponential
    const double sa = (a.s == 0.0) ? 0.0 : a.s * exp2((double)(a.m - r.m) * (double)it_log2e);
    const double sb = (b.s == 0.0) ? 0.0 : b.s * exp2((double)(b.m - r.m) * (double)it_log2e);
    r.s = sa + sb;
    return r;
}

__device__ __forceinline__ Red red_shfl_xor(const Red& a, int o) {
    Red r;
    r.m = __shfl_xor(a.m, o, kWave);
    r.am = __shfl_xor(a.am, o, kWave);
    r.s = __shfl_xor(a.s, o, kWave);
    return r;
}

template <bool kGreedy>
__device__ __forceinline__ void red_push(Red& r, float z, int v, float it_log2e) {
    if (z > r.m) {
        if (!kGreedy && r.s != 0.0) r.s *= exp2((double)(r.m - z) * (double)it_log2e);
        r.m = z;
        r.am = v;
    }
    if (!kGreedy) r.s += unnorm_prob(z, r.m, it_log2e);
}

// ---- 1. statistics -----------------------------------------------------------------------------------
template <bool kGreedy>
__global__ __launch_bounds__(kStatThreads) void accept_stats_kernel(AcceptArgs a) {
    const int split = blockIdx.x;
    const int mat = blockIdx.y / a.T;
    const int row = blockIdx.y % a.T;
    const int b = blockIdx.z;
    const float* base = (mat == 0 ? a.target : a.draft) + ((int64_t)b * a.T + row) * a.row_stride;
    const int begin = split * a.split_len;
    const int end = min(a.V, begin + a.split_len);
    const float it = kGreedy ? 0.f : kLog2e / a.temperature;

    Red r{-INFINITY, 0x7fffffff, 0.0};
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(base + begin) & 15) == 0);
    int v = begin;
    if (vec_ok) {
        const int n4 = (end - begin) / 4;
        const float4* b4 = reinterpret_cast<const float4*>(base + begin);
        for (int i = threadIdx.x; i < n4; i += kStatThreads) {
            const float4 x = b4[i];
            const int v0 = begin + 4 * i;
            const float mx = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
            if (mx > r.m) {
                if (!kGreedy && r.s != 0.0) r.s *= exp2((double)(r.m - mx) * (double)it);
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
        v = begin + 4 * n4;
    }
    for (int i = v + threadIdx.x; i < end; i += kStatThreads) red_push<kGreedy>(r, base[i], i, it);

#pragma unroll
    for (int o = 32; o > 0; o >>= 1) r = red_merge(r, red_shfl_xor(r, o), it);
    __shared__ Red wred[kStatThreads / kWave];
    if ((threadIdx.x & (kWave - 1)) == 0) wred[threadIdx.x / kWave] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
        Red t = wred[0];
        for (int w = 1; w < kStatThreads / kWave; ++w) t = red_merge(t, wred[w], it);
        RowStat* out = a.stats + ((((int64_t)b * a.n_mat + mat) * a.T + row) * a.splits + split);
        out->max_logit = t.m;
        out->argmax = t.am;
        out->sum_exp = t.s;
    }
}

// Merged statistics of one row, from its ranges.
__device__ __forceinline__ Red merged_row_stat(const AcceptArgs& a, int b, int mat, int row, float it) {
    const RowStat* st = a.stats + ((((int64_t)b * a.n_mat + mat) * a.T + row) * a.splits);
    Red t{st[0].max_logit, st[0].argmax, st[0].sum_exp};
    for (int s = 1; s < a.splits; ++s) {
        if (s * a.split_len >= a.V) break;
        t = red_merge(t, Red{st[s].max_logit, st[s].argmax, st[s].sum_exp}, it);
    }
    return t;
}

// ---- the law at a node after a number of rejections, one vocabulary entry at a time -------------------
struct ChainStep {        // what rejecting one child did to the laws
    int tok;              // the rejected token
    double inv_z;         // 1 / normaliser of max(p - q, 0)   (0 when the residual had no mass: p kept)
    double inv_qs;        // draft rule without replacement: 1 / (mass of q left after removing tok); else 1
    double inv_ps;        // deterministic rule: 1 / (mass of p left after removing tok)
};

template <int kRule>
__device__ __forceinline__ void law_after(int v, double p0, double q0, const ChainStep* steps, int n,
                                          double* p_out, double* q_out) {
    double p = p0, q = q0;
    for (int i = 0; i < n; ++i) {
        const ChainStep st = steps[i];
        if (kRule == TV_RULE_DETERMINISTIC) {
            p = (v == st.tok) ? 0.0 : ((st.inv_ps > 0.0) ? p * st.inv_ps : p);
        } else {
            const double r = fmax(p - q, 0.0);
            if (st.inv_z > 0.0) p = r * st.inv_z;
            if (kRule == TV_RULE_DRAFT_WOR) q = (v == st.tok) ? 0.0 : ((st.inv_qs > 0.0) ? q * st.inv_qs : q);
        }
    }
    *p_out = p;
    *q_out = q;
}

__device__ __forceinline__ double block_sum(double x, double* scratch /* kWalkWaves doubles */) {
    x = wave_sum(x);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[threadIdx.x / kWave] = x;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < (int)(blockDim.x / kWave); ++w) t += scratch[w];
    return t;
}

// ---- 2. sibling chains (draft rules) --------------------------------------------------------------------
template <int kRule>
__global__ __launch_bounds__(kWalkThreads) void accept_chain_kernel(AcceptArgs a) {
    const int u = blockIdx.x;
    const int b = blockIdx.y;
    const int T = a.T, V = a.V;
    __shared__ int s_parent[kMaxRows];
    __shared__ int s_token[kMaxRows];
    __shared__ int s_child[kMaxRows];
    __shared__ ChainStep s_steps[kMaxRows];
    __shared__ double s_red[kWalkWaves];
    __shared__ int s_flag, s_k;
    for (int i = threadIdx.x; i < T; i += blockDim.x) {
        s_parent[i] = a.parent[(int64_t)b * T + i];
        s_token[i] = a.token[(int64_t)b * T + i];
    }
    __syncthreads();
    int bad = validate_tree(s_parent, nullptr, T, &s_flag);
    if (threadIdx.x == 0) {
        int k = 0, tok_bad = 0;
        for (int c = 0; c < T; ++c) {
            if (s_token[c] < 0 || s_token[c] >= V) tok_bad = 1;
            if (c > u && s_parent[c] == u) s_child[k++] = c;
        }
        s_k = (tok_bad || bad) ? 0 : k;
    }
    __syncthreads();
    const int k = s_k;
    if (k == 0) return;     // leaf, or malformed input (the walk kernel reports it)

    const float it = kLog2e / a.temperature;
    const Red sp = merged_row_stat(a, b, 0, u, it);
    const Red sq = merged_row_stat(a, b, 1, u, it);
    const double inv_sp = 1.0 / sp.s, inv_sq = 1.0 / sq.s;
    const float* prow = a.target + ((int64_t)b * T + u) * a.row_stride;
    const float* qrow = a.draft + ((int64_t)b * T + u) * a.row_stride;

    for (int j = 0; j < k; ++j) {
        const int c = s_child[j];
        if (threadIdx.x == 0) {
            const int x = s_token[c];
            double p, q;
            law_after<kRule>(x, unnorm_prob(prow[x], sp.m, it) * inv_sp, unnorm_prob(qrow[x], sq.m, it) * inv_sq,
                             s_steps, j, &p, &q);
            const double uc = (double)a.uniforms[(int64_t)b * 2 * T + c];
            a.accept_bit[(int64_t)b * T + c] = (uc * q < p) ? 1 : 0;
            ChainStep st;
            st.tok = x;
            st.inv_z = 0.0;
            st.inv_ps = 1.0;
            const double qs = 1.0 - q;      // mass of q left once x is removed
            st.inv_qs = (kRule == TV_RULE_DRAFT_WOR && qs > 0.0) ? 1.0 / qs : 0.0;
            s_steps[j] = st;
        }
        __syncthreads();
        // normaliser of the corrected law after rejecting child j
        double part = 0.0;
        for (int v = threadIdx.x; v < V; v += blockDim.x) {
            double p, q;
            law_after<kRule>(v, unnorm_prob(prow[v], sp.m, it) * inv_sp, unnorm_prob(qrow[v], sq.m, it) * inv_sq,
                             s_steps, j, &p, &q);
            part += fmax(p - q, 0.0);
        }
        const double z = block_sum(part, s_red);
        if (threadIdx.x == 0) {
            s_steps[j].inv_z = (z > 0.0) ? 1.0 / z : 0.0;
            a.chain_z[(int64_t)b * T + c] = z;
        }
        __syncthreads();
    }
}

// ---- 3. walk + final draw ---------------------------------------------------------------------------------
struct WalkShared {
    int parent[kMaxRows];
    int token[kMaxRows];
    float unif[2 * kMaxRows];
    float m_p[kMaxRows];
    float m_q[kMaxRows];
    double inv_s_p[kMaxRows];
    double inv_s_q[kMaxRows];
    int argmax[kMaxRows];
    float z_tok_p[kMaxRows];      // target logit of node c's token in its parent's row
    float z_tok_q[kMaxRows];
    ChainStep steps[kMaxRows];
    double red[kWalkWaves];
    double wave_tot[kWalkWaves];
    double chunk_tot[2 * kWalkWaves];
    int last_pos[kWalkWaves];
    int flag, cur, n_steps, rejected_any, len, tok_out;
};

template <int kRule>
__device__ __forceinline__ double final_law(const AcceptArgs& a, const WalkShared& sh, const float* prow,
                                            const float* qrow, int node, int v, float it) {
    const double p0 = unnorm_prob(prow[v], sh.m_p[node], it) * sh.inv_s_p[node];
    double q0 = 0.0;
    if (kRule == TV_RULE_DRAFT_WOR || kRule == TV_RULE_DRAFT_WR)
        q0 = unnorm_prob(qrow[v], sh.m_q[node], it) * sh.inv_s_q[node];
    double p, q;
    law_after<kRule>(v, p0, q0, sh.steps, sh.n_steps, &p, &q);
    return p;
}

template <int kRule>
__global__ __launch_bounds__(kWalkThreads) void accept_walk_kernel(AcceptArgs a) {
    const int b = blockIdx.x;
    const int T = a.T, V = a.V;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr bool kGreedy = (kRule == TV_RULE_GREEDY);
    constexpr bool kDraft = (kRule == TV_RULE_DRAFT_WOR || kRule == TV_RULE_DRAFT_WR);
    __shared__ WalkShared sh;
    const float it = kGreedy ? 0.f : kLog2e / a.temperature;

    for (int i = tid; i < T; i += blockDim.x) {
        sh.parent[i] = a.parent[(int64_t)b * T + i];
        sh.token[i] = a.token[(int64_t)b * T + i];
        if (!kGreedy) {
            sh.unif[i] = a.uniforms[(int64_t)b * 2 * T + i];
            sh.unif[T + i] = a.uniforms[(int64_t)b * 2 * T + T + i];
        }
    }
    __syncthreads();
    int bad = validate_tree(sh.parent, nullptr, T, &sh.flag);
    {
        int tok_bad = 0;
        for (int i = tid; i < T; i += blockDim.x)
            if (sh.token[i] < 0 || sh.token[i] >= V) tok_bad = 1;
        if (tok_bad) atomicOr(&sh.flag, TV_STATUS_BAD_TOKEN);
        __syncthreads();
        bad = sh.flag;
    }
    int32_t* path = a.path + (int64_t)b * T;
    if (bad) {
        for (int i = tid; i < T; i += blockDim.x) path[i] = -1;
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

    // per-row statistics and each node's token logit in its parent's row
    for (int i = tid; i < T; i += blockDim.x) {
        const Red sp = merged_row_stat(a, b, 0, i, it);
        sh.m_p[i] = sp.m;
        sh.argmax[i] = sp.am;
        sh.inv_s_p[i] = kGreedy ? 0.0 : 1.0 / sp.s;
        if (kDraft) {
            const Red sq = merged_row_stat(a, b, 1, i, it);
            sh.m_q[i] = sq.m;
            sh.inv_s_q[i] = 1.0 / sq.s;
        }
        if (i > 0 && !kGreedy) {
            const int64_t r = ((int64_t)b * T + sh.parent[i]) * a.row_stride + sh.token[i];
            sh.z_tok_p[i] = a.target[r];
        }
    }
    __syncthreads();

    // the walk: one thread, LDS only
    if (tid == 0) {
        int cur = 0, len = 0, nrej = 0;
        path[0] = 0;
        for (;;) {
            nrej = 0;
            int next = -1;
            for (int c = cur + 1; c < T; ++c) {
                if (sh.parent[c] != cur) continue;
                const int x = sh.token[c];
                bool acc;
                if (kGreedy) {
                    acc = (x == sh.argmax[cur]);
                } else if (kRule == TV_RULE_DETERMINISTIC) {
                    double p, q;
                    law_after<kRule>(x, unnorm_prob(sh.z_tok_p[c], sh.m_p[cur], it) * sh.inv_s_p[cur], 0.0,
                                     sh.steps, nrej, &p, &q);
                    acc = ((double)sh.unif[c] < p);
                    if (!acc) {
                        const double ps = 1.0 - p;       // mass of p left once x is removed
                        sh.steps[nrej] = ChainStep{x, 0.0, 0.0, (ps > 0.0) ? 1.0 / ps : 0.0};
                    }
                } else {
                    acc = (a.accept_bit[(int64_t)b * T + c] != 0);
                    if (!acc) {
                        // rebuild the chain step exactly as the chain kernel formed it
                        double p, q;
                        const int64_t r = ((int64_t)b * T + cur) * a.row_stride + x;
                        law_after<kRule>(x, unnorm_prob(sh.z_tok_p[c], sh.m_p[cur], it) * sh.inv_s_p[cur],
                                         unnorm_prob(a.draft[r], sh.m_q[cur], it) * sh.inv_s_q[cur],
                                         sh.steps, nrej, &p, &q);
                        const double z = a.chain_z[(int64_t)b * T + c];
                        const double qs = 1.0 - q;
                        sh.steps[nrej] = ChainStep{x, (z > 0.0) ? 1.0 / z : 0.0,
                                                   (kRule == TV_RULE_DRAFT_WOR && qs > 0.0) ? 1.0 / qs : 0.0, 1.0};
                    }
                }
                if (acc) { next = c; break; }
                ++nrej;
            }
            if (next < 0) break;
            cur = next;
            path[++len] = cur;
        }
        for (int i = len + 1; i < T; ++i) path[i] = -1;
        sh.cur = cur;
        sh.len = len;
        sh.n_steps = nrej;
        sh.rejected_any = (nrej > 0);
        sh.tok_out = -1;
    }
    __syncthreads();
    const int cur = sh.cur;

    if (kGreedy) {
        if (tid == 0) sh.tok_out = sh.argmax[cur];
    } else {
        // ---- inverse CDF at the stop node: first v whose running sum of the law exceeds u --------
        const float* prow = a.target + ((int64_t)b * T + cur) * a.row_stride;
        const float* qrow = kDraft ? a.draft + ((int64_t)b * T + cur) * a.row_stride : nullptr;
        const double u = (double)sh.unif[T + cur];
        // level 1: each wave owns a contiguous range (a multiple of 256 entries)
        const int per_wave = ((V + kWalkWaves - 1) / kWalkWaves + 255) / 256 * 256;
        {
            const int lo = wave * per_wave, hi = min(V, lo + per_wave);
            double acc = 0.0;
            int last = -1;
#pragma unroll 4
            for (int v = lo + lane; v < hi; v += kWave) {
                const double pv = final_law<kRule>(a, sh, prow, qrow, cur, v, it);
                acc += pv;
                if (pv > 0.0) last = v;
            }
            acc = wave_sum(acc);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o, kWave));
            if (lane == 0) { sh.wave_tot[wave] = acc; sh.last_pos[wave] = last; }
        }
        __syncthreads();
        int w_star = -1;
        double base = 0.0;
        for (int w = 0; w < kWalkWaves; ++w) {
            if (base + sh.wave_tot[w] > u) { w_star = w; break; }
            base += sh.wave_tot[w];
        }
        if (w_star < 0) {
            // rounding left the total at or below u: the last entry that carries mass
            if (tid == 0) {
                int last = -1;
                for (int w = 0; w < kWalkWaves; ++w) last = max(last, sh.last_pos[w]);
                sh.tok_out = last;
            }
        } else {
            // level 2: the chosen range is cut into at most 2*kWalkWaves chunks, two per wave
            const int lo = w_star * per_wave, hi = min(V, lo + per_wave);
            const int chunk_len = ((per_wave + 2 * kWalkWaves - 1) / (2 * kWalkWaves) + kWave - 1) / kWave * kWave;
            const int n_chunks = (hi - lo + chunk_len - 1) / chunk_len;      // <= 2*kWalkWaves
            for (int ch = wave; ch < n_chunks; ch += kWalkWaves) {
                double acc = 0.0;
                const int c_lo = lo + ch * chunk_len, c_hi = min(hi, c_lo + chunk_len);
                for (int v = c_lo + lane; v < c_hi; v += kWave) acc += final_law<kRule>(a, sh, prow, qrow, cur, v, it);
                acc = wave_sum(acc);
                if (lane == 0) sh.chunk_tot[ch] = acc;
            }
            __syncthreads();
            int c_star = -1;
            for (int ch = 0; ch < n_chunks; ++ch) {
                if (base + sh.chunk_tot[ch] > u) { c_star = ch; break; }
                base += sh.chunk_tot[ch];
            }
            // level 3: one wave scans the chosen chunk in vocabulary order
            if (wave == 0) {
                // (if rounding hid the crossing from the chunk sums, the whole range is scanned)
                const int s_lo = (c_star >= 0) ? lo + c_star * chunk_len : lo;
                const int s_hi = (c_star >= 0) ? min(hi, s_lo + chunk_len) : hi;
                double run = base;
                int found = -1;
                for (int v0 = s_lo; v0 < s_hi && found < 0; v0 += kWave) {
                    const int v = v0 + lane;
                    const double pv = (v < s_hi) ? final_law<kRule>(a, sh, prow, qrow, cur, v, it) : 0.0;
                    double inc = pv;           // inclusive scan over the wave, in vocabulary order
#pragma unroll
                    for (int o = 1; o < kWave; o <<= 1) {
                        const double t = __shfl_up(inc, o, kWave);
                        if (lane >= o) inc += t;
                    }
                    const unsigned long long hit = __ballot((run + inc > u) && v < s_hi);
                    if (hit) found = v0 + __ffsll((long long)hit) - 1;
                    run += __shfl(inc, kWave - 1, kWave);
                }
                if (lane == 0) {
                    if (found < 0) {
                        // the chunk sums said the crossing is here, the in-order sums round just below:
                        // take the last entry of the scanned span that carries mass
                        for (int v = s_hi - 1; v >= s_lo && found < 0; --v)
                            if (final_law<kRule>(a, sh, prow, qrow, cur, v, it) > 0.0) found = v;
                    }
                    sh.tok_out = found;
                }
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        a.status[b] = TV_STATUS_OK;
        a.n_accepted[b] = sh.len;
        a.final_token[b] = sh.tok_out;
        a.final_kind[b] = sh.rejected_any ? TV_FINAL_RESIDUAL : TV_FINAL_BONUS;
        a.last_node[b] = cur;
        if (a.selected_con) {
            int sel = -1;
            if (a.con_anchor)
                for (int c = 0; c < a.C && sel < 0; ++c)
                    if (a.con_anchor[(int64_t)b * a.C + c] == cur) sel = c;
            a.selected_con[b] = sel;
        }
    }
}

}  // namespace

int plan_accept(const tv_accept_desc& d, AcceptPlan* plan) {
    AcceptPlan p{};
    p.n_mat = (d.rule == TV_RULE_DRAFT_WOR || d.rule == TV_RULE_DRAFT_WR) ? 2 : 1;
    // enough workgroups to fill 256 CUs a few times over, ranges no shorter than 4096 entries
    const int rows = d.B * d.T * p.n_mat;
    int splits = (2048 + rows - 1) / rows;
    const int max_splits = (d.V + 4095) / 4096;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    int len = (d.V + splits - 1) / splits;
    len = (len + 3) / 4 * 4;
    p.splits = (d.V + len - 1) / len;
    p.split_len = len;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    p.stats_bytes = up((size_t)rows * p.splits * sizeof(RowStat));
    p.chain_bytes = up((size_t)d.B * d.T * sizeof(double));
    p.bits_bytes = up((size_t)d.B * d.T * sizeof(int32_t));
    p.total_bytes = p.stats_bytes + p.chain_bytes + p.bits_bytes;
    *plan = p;
    return TV_OK;
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t s) {
    const dim3 gs(a.splits, a.T * a.n_mat, a.B);
    if (a.rule == TV_RULE_GREEDY) accept_stats_kernel<true><<<gs, kStatThreads, 0, s>>>(a);
    else accept_stats_kernel<false><<<gs, kStatThreads, 0, s>>>(a);
    if (a.rule == TV_RULE_DRAFT_WOR) accept_chain_kernel<TV_RULE_DRAFT_WOR><<<dim3(a.T, a.B), kWalkThreads, 0, s>>>(a);
    else if (a.rule == TV_RULE_DRAFT_WR) accept_chain_kernel<TV_RULE_DRAFT_WR><<<dim3(a.T, a.B), kWalkThreads, 0, s>>>(a);
    switch (a.rule) {
        case TV_RULE_GREEDY: accept_walk_kernel<TV_RULE_GREEDY><<<a.B, kWalkThreads, 0, s>>>(a); break;
        case TV_RULE_DETERMINISTIC: accept_walk_kernel<TV_RULE_DETERMINISTIC><<<a.B, kWalkThreads, 0, s>>>(a); break;
        case TV_RULE_DRAFT_WOR: accept_walk_kernel<TV_RULE_DRAFT_WOR><<<a.B, kWalkThreads, 0, s>>>(a); break;
        default: accept_walk_kernel<TV_RULE_DRAFT_WR><<<a.B, kWalkThreads, 0, s>>>(a); break;
    }
    return hipGetLastError();
}

}  // namespace tv
