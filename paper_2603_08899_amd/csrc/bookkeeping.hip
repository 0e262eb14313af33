// The two small steps around the verification pass, for gfx950:
//   tree_commit        moves the K/V rows of the accepted path to the front of this step's rows in every
//                      layer's pool (rejected nodes and contemplate rows are dropped) and picks the future
//                      prediction of the last accepted token   (paper: Section 2, step 3; Section 3.1)
//   contemplate_embed  mixture-of-experts embedding of a contemplate / future token: router logits,
//                      softmax, top-K, weighted sum of expert embeddings   (paper: Section 3.2)
// Both are small and bound by memory latency; plain ALUs, 16-byte accesses.  The embedding runs as two
// kernels: one router logit per workgroup, then one block of output columns per workgroup.
#include "tv_internal.hpp"

namespace tv {

namespace {

constexpr int kCommitThreads = 256;
constexpr int kCommitHeld = 8;                                  // 16-byte pieces a lane holds at once
constexpr int kCommitChunk = kCommitThreads * kCommitHeld;      // pieces moved between two barriers

// ---- tree_commit ------------------------------------------------------------------------------------------
// Grid (n_layers, B, 2): one workgroup moves the accepted rows of one sequence in the K (z = 0) or V (z = 1)
// pool of one layer.  Row j of the new cache comes from new row src[j] >= j; several moves of one sequence
// overlap (a destination may be the source of an earlier entry of the path), so a chunk of rows is read
// completely before any of it is written.  Later sources lie strictly behind every earlier destination, so
// chunks can follow each other without further ordering.
// What the first loads hang on comes as leading scalar arguments (in registers when a wave starts); the argument
// struct is read behind them.  The per-sequence scalars and the whole path are requested at once - the path
// before its length is known - so that the kernel pays one memory round trip for them, one for the row map (if
// there is one) and one for the rows.
struct CommitKernArgs {
    const int32_t* n_accepted;
    const int32_t* path;
    const int32_t* prefix_len;
    const int64_t* kv_offset;
    const int32_t* selected_con;
    int T;
    CommitArgs a;
};
static_assert(offsetof(CommitKernArgs, a) == 48, "kernel-argument layout of commit_kernel");

__device__ __forceinline__ void global_pointers(CommitArgs& a) {
    a.k = global_pointer(a.k);
    a.v = global_pointer(a.v);
    a.node_row = global_pointer(a.node_row);
    a.hidden = global_pointer(a.hidden);
    a.con_row = global_pointer(a.con_row);
    a.f_out = global_pointer(a.f_out);
    a.new_prefix_len = global_pointer(a.new_prefix_len);
    a.status = global_pointer(a.status);
}

__global__ __launch_bounds__(kCommitThreads) void commit_kernel(const int32_t* n_accepted, const int32_t* path_in,
                                                                const int32_t* prefix_len, const int64_t* kv_offset,
                                                                const int32_t* selected_con, int T,
                                                                CommitArgs /* read below */) {
    const int l = blockIdx.x, b = blockIdx.y, which = blockIdx.z;
    const int tid = threadIdx.x;
    __shared__ int s_src[kMaxRows];
    __shared__ int s_ok;
    const int n = n_accepted[b];
    const int P = prefix_len[b];
    const int64_t kv_first = kv_offset[b];
    const bool gathers_f = (l == 0 && which == 1);
    const int sel = (gathers_f && selected_con) ? selected_con[b] : -1;      // (null: nothing to gather)
    int node = -1, prev = -1;
    if (tid < T) {                       // (the path array has T entries whatever its length)
        node = path_in[(int64_t)b * T + tid];
        prev = (tid > 0) ? path_in[(int64_t)b * T + tid - 1] : -1;
    }
    CommitArgs a = kernarg_block_after_requests<CommitArgs>(offsetof(CommitKernArgs, a));
    global_pointers(a);
    // (the workgroup that gathers f fetches every contemplate row's index now, not only the selected one's once
    //  that is known: one round trip less in front of the copy)
    __shared__ int s_con[kMaxRows];
    if (gathers_f && a.hidden && tid < a.C && tid < kMaxRows) s_con[tid] = a.con_row[(int64_t)b * a.C + tid];
    if (tid == 0) s_ok = 1;
    __syncthreads();
    if (n >= 0 && n < T && tid <= n) {
        bool bad = node < 0 || node >= T || node <= prev || (tid == 0 && node != 0);
        int row = -1;
        if (!bad) {
            row = a.node_row ? a.node_row[(int64_t)b * T + node] : node;
            bad = row < 0 || row >= a.M;
        }
        s_src[tid] = row;
        if (bad) s_ok = 0;
    }
    __syncthreads();
    // the rows of the path must increase with it: the chunked move below relies on every source lying at or behind
    // its destination (row of entry j >= j)
    if (n >= 0 && n < T && tid >= 1 && tid <= n && s_src[tid] <= s_src[tid - 1]) s_ok = 0;
    __syncthreads();
    const bool ok = n >= 0 && n < T && s_ok != 0;
    if (l == 0 && which == 0 && tid == 0) {
        a.status[b] = (n >= 0 && !ok) ? TV_STATUS_BAD_PATH : TV_STATUS_OK;
        a.new_prefix_len[b] = P + (ok ? n + 1 : 0);
    }
    if (gathers_f && a.hidden) {
        // the future prediction that belongs to the last accepted token
        const int c = sel;
        const int row = (c >= 0 && c < a.C) ? (c < kMaxRows ? s_con[c] : a.con_row[(int64_t)b * a.C + c]) : -1;
        const int pieces = a.d_model * a.elem / 16;
        uint4* dst = reinterpret_cast<uint4*>(static_cast<unsigned char*>(a.f_out) + (int64_t)b * a.d_model * a.elem);
        const uint4* src = (row >= 0 && row < a.M)
            ? reinterpret_cast<const uint4*>(static_cast<const unsigned char*>(a.hidden) +
                                             ((int64_t)b * a.M + row) * a.d_model * a.elem)
            : nullptr;
        for (int i = tid; i < pieces; i += kCommitThreads) dst[i] = src ? src[i] : make_uint4(0u, 0u, 0u, 0u);
    }
    if (!ok) return;

    unsigned char* pool = static_cast<unsigned char*>(which ? a.v : a.k) +
                          ((int64_t)l * a.layer_stride + (kv_first + P) * a.tok_stride) * a.elem;
    const int segs = a.D * a.elem / 16;                 // 16-byte pieces of one head's row
    const int per_row = a.Hkv * segs;
    auto piece = [&](int row, int rem) -> uint4* {
        const int g = rem / segs, sg = rem - g * segs;
        return reinterpret_cast<uint4*>(pool + ((int64_t)row * a.tok_stride + (int64_t)g * a.head_stride) * a.elem) + sg;
    };
    if (per_row <= kCommitChunk) {
        const int rows_per_chunk = kCommitChunk / per_row;
        for (int j0 = 0; j0 <= n; j0 += rows_per_chunk) {
            const int rows = min(rows_per_chunk, n + 1 - j0);
            const int units = rows * per_row;
            uint4 held[kCommitHeld];
#pragma unroll
            for (int k = 0; k < kCommitHeld; ++k) {
                const int u = tid + k * kCommitThreads;
                if (u < units) {
                    const int j = j0 + u / per_row;
                    held[k] = *piece(s_src[j], u % per_row);
                }
            }
            __syncthreads();                            // every read of the chunk is complete
#pragma unroll
            for (int k = 0; k < kCommitHeld; ++k) {
                const int u = tid + k * kCommitThreads;
                if (u < units) {
                    const int j = j0 + u / per_row;
                    if (s_src[j] != j) *piece(j, u % per_row) = held[k];
                }
            }
        }
    } else {
        // very wide rows: one row at a time (its source is another row, or itself)
        for (int j = 0; j <= n; ++j) {
            if (s_src[j] == j) continue;
            for (int u = tid; u < per_row; u += kCommitThreads) *piece(j, u) = *piece(s_src[j], u);
            __syncthreads();
        }
    }
}

// ---- contemplate_embed --------------------------------------------------------------------------------------
constexpr int kEmbedThreads = 256;
constexpr int kEmbedWaves = kEmbedThreads / kWave;
constexpr int kEmbedCols = kEmbedThreads * 8;        // output columns per workgroup of the second kernel
constexpr int kMaxExperts = 64;

template <bool kBf16>
__device__ __forceinline__ void load8(const void* base, int64_t index, float* x) {
    if (kBf16) {
        const uint4 r = *reinterpret_cast<const uint4*>(static_cast<const unsigned short*>(base) + index);
        const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        const float4 r0 = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + index);
        const float4 r1 = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + index + 4);
        x[0] = r0.x; x[1] = r0.y; x[2] = r0.z; x[3] = r0.w;
        x[4] = r1.x; x[5] = r1.y; x[6] = r1.z; x[7] = r1.w;
    }
}

// Kernel 1, grid (n_expert, B): one router logit per workgroup (fp32 dot product, a lane covers 8 consecutive
// inputs per step; lanes, then waves, are summed in a fixed order).
template <bool kBf16>
__global__ __launch_bounds__(kEmbedThreads) void embed_logit_kernel(EmbedArgs a) {
    const int e = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    __shared__ float s_part[kEmbedWaves];
    float acc = 0.f;
    for (int i = tid * 8; i < a.d_in; i += kEmbedThreads * 8) {
        float hv[8], wv[8];
        load8<kBf16>(a.h, (int64_t)b * a.d_in + i, hv);
        load8<kBf16>(a.router_w, (int64_t)e * a.d_in + i, wv);
#pragma unroll
        for (int x = 0; x < 8; ++x) acc = fmaf(hv[x], wv[x], acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) s_part[wave] = acc;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < kEmbedWaves; ++w) t += s_part[w];
        a.logits[(int64_t)b * a.n_expert + e] = t;
    }
}

// Kernel 2, grid (column blocks, B): every workgroup normalises the (at most 64) logits and selects the K best
// experts itself (lowest index on ties, best first), then forms its block of output columns.
template <bool kBf16>
__global__ __launch_bounds__(kEmbedThreads) void embed_mix_kernel(EmbedArgs a) {
    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    __shared__ float s_gate[kMaxExperts];
    __shared__ int s_chosen[kMaxExperts];
    if (wave == 0) {
        const bool live = lane < a.n_expert;
        const float z = live ? a.logits[(int64_t)b * a.n_expert + lane] : -INFINITY;
        const float m = wave_max(z);
        const float ex = live ? expf(z - m) : 0.f;
        const float g = ex / wave_sum(ex);
        const bool writer = (blockIdx.x == 0);
        if (live) {
            s_gate[lane] = g;
            if (writer && a.gates) a.gates[(int64_t)b * a.n_expert + lane] = g;
        }
        float cand = live ? g : -1.f;
        for (int r = 0; r < a.k_expert; ++r) {
            float bv = cand;
            int bi = lane;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(bv, o, kWave);
                const int oi = __shfl_xor(bi, o, kWave);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (lane == 0) {
                s_chosen[r] = bi;
                if (writer && a.chosen) a.chosen[(int64_t)b * a.k_expert + r] = bi;
            }
            if (lane == bi) cand = -1.f;
        }
    }
    __syncthreads();

    // out = sum over the chosen experts of gate * embedding
    const int c = blockIdx.x * kEmbedCols + tid * 8;
    if (c >= a.d_out) return;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < a.k_expert; ++r) {
        const int e = s_chosen[r];
        const float g = s_gate[e];
        float ev[8];
        load8<kBf16>(a.expert_emb, (int64_t)e * a.d_out + c, ev);
#pragma unroll
        for (int x = 0; x < 8; ++x) acc[x] = fmaf(g, ev[x], acc[x]);
    }
    if (kBf16) {
        typedef __bf16 bf16x8 __attribute__((ext_vector_type(8), may_alias));
        bf16x8 o;
#pragma unroll
        for (int x = 0; x < 8; ++x) o[x] = (__bf16)acc[x];
        *reinterpret_cast<bf16x8*>(static_cast<unsigned short*>(a.out) + (int64_t)b * a.d_out + c) = o;
    } else {
        float* o = static_cast<float*>(a.out) + (int64_t)b * a.d_out + c;
        *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

}  // namespace

hipError_t launch_commit(const CommitArgs& a, hipStream_t s) {
    commit_kernel<<<dim3(a.n_layers, a.B, 2), kCommitThreads, 0, s>>>(a.n_accepted, a.path, a.prefix_len, a.kv_offset,
                                                                    a.selected_con, a.T, a);
    return hipGetLastError();
}

hipError_t launch_embed(const EmbedArgs& a, hipStream_t s) {
    const dim3 g1(a.n_expert, a.B), g2((a.d_out + kEmbedCols - 1) / kEmbedCols, a.B);
    if (a.bf16) {
        embed_logit_kernel<true><<<g1, kEmbedThreads, 0, s>>>(a);
        embed_mix_kernel<true><<<g2, kEmbedThreads, 0, s>>>(a);
    } else {
        embed_logit_kernel<false><<<g1, kEmbedThreads, 0, s>>>(a);
        embed_mix_kernel<false><<<g2, kEmbedThreads, 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace tv
