// Internal declarations shared by the translation units of libconfu_verify.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "confu_verify.h"

namespace tv {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kMaxRows = TV_MAX_ROWS;
constexpr int kMaskWords = 2;        // 64-bit words of ancestor mask per row (M <= 128)

// ---- attention plan: how one call is cut into workgroups -------------------------------------
struct AttnPlan {
    int G;                 // query heads per KV head
    int row_blocks;        // 64-row blocks of the G*M packed rows of one KV head (bf16 path), padded to a multiple of rb_per_wg
    int rb_per_wg;         // 64-row blocks covered by one workgroup: 1, 2 or 4
    int n_chunks;          // key ranges the (prefix + new rows) of a sequence are cut into
    size_t part_o_bytes;   // workspace: partial outputs
    size_t part_ml_bytes;  // workspace: partial (max, sum) pairs
    size_t total_bytes;
};

int plan_attention(const tv_attn_desc& d, AttnPlan* plan);

// A kernel's by-value argument struct, read through a pointer the compiler cannot look through: none of its loads
// moves above the call, i.e. above the requests a kernel has issued from its leading scalar arguments (those are in
// registers when a wave starts - kernel-argument preload, see the build flags - while the rest of the argument
// segment costs a memory round trip, which then runs under the requests' own instead of in front of them).
// `offset`: byte offset of the struct in the kernel-argument segment (arguments in order, natural alignment).
// A pointer that came out of such a struct is a plain (generic) pointer to the compiler; this says again that it
// points to global memory, so that accesses through it are global loads and stores, not flat ones.
template <typename T>
__device__ __forceinline__ T* global_pointer(T* p) {
    typedef T __attribute__((address_space(1)))* global_ptr;
    return (T*)(global_ptr)(uintptr_t)p;          // (through the address value: a cast between pointers alone is dropped)
}
template <typename Block>
__device__ __forceinline__ Block kernarg_block_after_requests(unsigned offset) {
    typedef const unsigned char __attribute__((address_space(4)))* kernarg_bytes;
    typedef const unsigned __attribute__((address_space(4)))* kernarg_words;
    static_assert(sizeof(Block) % 4 == 0 && alignof(Block) <= 8, "copied word by word");
    kernarg_bytes ka = (kernarg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ka) : : "memory");
    kernarg_words src = (kernarg_words)(ka + offset);
    Block blk;
    unsigned* dst = reinterpret_cast<unsigned*>(&blk);
#pragma unroll
    for (unsigned w = 0; w < sizeof(Block) / 4; ++w) dst[w] = src[w];
    return blk;
}

struct AttnArgs {
    const void* q;
    const void* k;
    const void* v;
    const int64_t* kv_offset;
    const int32_t* prefix_len;
    const int32_t* parent;
    const uint8_t* kind;
    const unsigned char* prepared;     // [B] PreparedTree records written by tv_prepare_tree, or null
    void* out;
    float* lse;
    int32_t* status;
    void* part_o;      // partial outputs, bf16, each already divided by its own sum
    float* part_ml;
    int B, M, Hq, Hkv, D, G;
    int soft_len, max_prefix_len;
    float scale;
    float inv_M;                       // 1 / M
    int64_t tok_stride, head_stride;   // elements
    int row_blocks, n_chunks, rb_per_wg;
};

// What tv_prepare_tree leaves per sequence: the ancestor mask of every row (Section 3.1 / Figure 4: one mask per
// verification step, shared by all layers), the row kinds, and the verdict of the tree checks.
struct PreparedTree {
    unsigned long long bits[kMaxRows][2];   // zeros when the tree is malformed
    unsigned char kind[kMaxRows];
    int32_t status;                         // TV_STATUS_BAD_PARENT / TV_STATUS_BAD_KIND bits
    unsigned char pad[TV_PREPARED_TREE_BYTES - kMaxRows * 16 - kMaxRows - 4];
};
static_assert(sizeof(PreparedTree) == TV_PREPARED_TREE_BYTES, "record size is part of the ABI");

hipError_t launch_prepare_tree(const int32_t* parent, const uint8_t* kind, int B, int M, PreparedTree* out, hipStream_t s);
hipError_t launch_attention_f32(const AttnArgs& a, hipStream_t s);
hipError_t launch_attention_bf16(const AttnArgs& a, hipStream_t s);

// ---- acceptance ---------------------------------------------------------------------------------
struct RowStat {          // softmax statistics of one range of one logits row
    float  max_logit;     // max z over the range
    int    argmax;        // lowest index attaining it
    double sum_exp;       // sum exp((z - max_logit) / temperature) over the range
};

struct AcceptPlan {
    int splits;           // ranges a logits row is cut into for the statistics pass (<= 256)
    int split_len;        // elements per range (multiple of 8)
    int n_mat;            // 1 (target only) or 2 (target and draft)
    int chain_slices;     // draft rules: workgroups per node in the sibling-chain kernel
    size_t stats_bytes, ztok_bytes, chain_bytes, bits_bytes, chain_parts_bytes, total_bytes;
};

int plan_accept(const tv_accept_desc& d, AcceptPlan* plan);

struct AcceptArgs {
    const void* target;   // [B][T] rows of V logits, row_stride elements apart: fp32, or bf16 when logits_bf16
    const void* draft;
    int logits_bf16;
    const int32_t* token;
    const int32_t* parent;
    const float* uniforms;
    const int32_t* con_anchor;
    int32_t* path;
    int32_t* n_accepted;
    int32_t* final_token;
    int32_t* final_kind;
    int32_t* last_node;
    int32_t* selected_con;
    int32_t* status;
    RowStat* stats;       // [B][n_mat][T][splits]
    float*   z_tok;       // [B][n_mat][T]: logit of node c's token in its parent's row
    double*  chain_z;     // [B][T]: normaliser of the corrected law after rejecting child c
    int32_t* accept_bit;  // [B][T] (draft rules)
    int32_t* sampled;     // [B][T] (sample-and-match rule; same storage as accept_bit): the target's token at each node
    unsigned long long* chain_parts;  // [B][T][chain_slices]: per child, every slice's share of its chain normaliser
                             // (fp64 bits; the two lowest are a tag: 0 = published, 3 = not yet)
    int B, T, V, C, rule;
    float temperature;
    int64_t row_stride;
    int splits, split_len, n_mat;
    int chain_slices;
    unsigned wait_limit;     // looks at another workgroup's slot before a workgroup computes that share itself
};

hipError_t launch_accept(const AcceptArgs& a, hipStream_t s);

// ---- commit of the accepted path, contemplate embedding ---------------------------------------------
struct CommitArgs {
    void* k;
    void* v;
    const int64_t* kv_offset;
    const int32_t* prefix_len;
    const int32_t* path;
    const int32_t* n_accepted;
    const int32_t* node_row;
    const void* hidden;
    const int32_t* con_row;
    const int32_t* selected_con;
    void* f_out;
    int32_t* new_prefix_len;
    int32_t* status;
    int B, T, M, Hkv, D, n_layers, C, d_model;
    int elem;                          // bytes per element
    int64_t layer_stride, tok_stride, head_stride;   // elements
};

struct EmbedArgs {
    const void* h;
    const void* router_w;
    const void* expert_emb;
    void* out;
    float* gates;
    int32_t* chosen;
    float* logits;                     // workspace [B][n_expert]
    int B, d_in, d_out, n_expert, k_expert;
    bool bf16;
};

hipError_t launch_commit(const CommitArgs& a, hipStream_t s);
hipError_t launch_embed(const EmbedArgs& a, hipStream_t s);

// ---- small device helpers -------------------------------------------------------------------------
// Wave-wide reductions with data-parallel-primitive moves (no LDS crossbar round trips, which a butterfly of six
// dependent shuffles pays one after the other): an inclusive scan - Hillis-Steele inside each row of 16 lanes, then
// lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3 - leaves the result in lane 63, which
// every lane then reads.  All lanes get the same bits.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int dpp_int(int old, int x) {
    return __builtin_amdgcn_update_dpp(old, x, kCtrl, kRowMask, 0xf, false);      // lanes without a source keep `old`
}
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_or_zero(float x) { return __int_as_float(dpp_int<kCtrl, kRowMask>(0, __float_as_int(x))); }
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_or_self(float x) {
    return __int_as_float(dpp_int<kCtrl, kRowMask>(__float_as_int(x), __float_as_int(x)));
}
template <int kCtrl, int kRowMask>
__device__ __forceinline__ double dpp_or_zero(double x) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    const unsigned lo = (unsigned)dpp_int<kCtrl, kRowMask>(0, (int)(unsigned)b);
    const unsigned hi = (unsigned)dpp_int<kCtrl, kRowMask>(0, (int)(unsigned)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ float last_lane(float x) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), kWave - 1)); }
__device__ __forceinline__ double last_lane(double x) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, kWave - 1);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), kWave - 1);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// inclusive prefix sums over the lanes of a wave (lane l: x of lanes 0 .. l, added in that association)
template <typename T>
__device__ __forceinline__ T wave_prefix_sum(T x) {
    x += dpp_or_zero<0x111, 0xf>(x);      // row_shr:1
    x += dpp_or_zero<0x112, 0xf>(x);      // row_shr:2
    x += dpp_or_zero<0x114, 0xf>(x);      // row_shr:4
    x += dpp_or_zero<0x118, 0xf>(x);      // row_shr:8
    x += dpp_or_zero<0x142, 0xa>(x);      // row_bcast:15 into rows 1 and 3
    x += dpp_or_zero<0x143, 0xc>(x);      // row_bcast:31 into rows 2 and 3
    return x;
}
__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_or_self<0x111, 0xf>(x));
    x = fmaxf(x, dpp_or_self<0x112, 0xf>(x));
    x = fmaxf(x, dpp_or_self<0x114, 0xf>(x));
    x = fmaxf(x, dpp_or_self<0x118, 0xf>(x));
    x = fmaxf(x, dpp_or_self<0x142, 0xa>(x));
    x = fmaxf(x, dpp_or_self<0x143, 0xc>(x));
    return last_lane(x);
}
__device__ __forceinline__ float wave_sum(float x) { return last_lane(wave_prefix_sum(x)); }
__device__ __forceinline__ double wave_sum(double x) { return last_lane(wave_prefix_sum(x)); }

// Validates one sequence's parent/kind arrays (already in LDS) with the whole workgroup and
// returns the TV_STATUS_* bits to every thread.  `flag` is one LDS word.
__device__ __forceinline__ int validate_tree(const int* parent, const unsigned char* kind, int M,
                                             int* flag) {
    if (threadIdx.x == 0) *flag = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < M; i += blockDim.x) {
        int bad = 0;
        const int p = parent[i];
        if (p < -1 || p >= i) bad |= TV_STATUS_BAD_PARENT;
        if (kind) {
            const int ki = kind[i];
            if (ki != TV_KIND_NODE && ki != TV_KIND_CONTEMPLATE) bad |= TV_STATUS_BAD_KIND;
            if (p >= 0 && p < i && ki == TV_KIND_NODE && kind[p] == TV_KIND_CONTEMPLATE) bad |= TV_STATUS_BAD_KIND;
        } else if (i > 0 && p < 0) {
            bad |= TV_STATUS_BAD_PARENT;       // acceptance trees have exactly one root
        }
        if (bad) atomicOr(flag, bad);
    }
    __syncthreads();
    return *flag;
}

// Ancestor-closure mask of row i: bit j set iff j is i or one of its ancestors.  parent[] must
// have passed validate_tree (parent[j] < j), so the walk ends within M steps.
__device__ __forceinline__ void ancestor_bits(const int* parent, int i, unsigned long long* w0,
                                              unsigned long long* w1) {
    unsigned long long a = 0, b = 0;
    int j = i;
    while (j >= 0) {
        if (j < 64) a |= 1ull << j; else b |= 1ull << (j - 64);
        j = parent[j];
    }
    *w0 = a;
    *w1 = b;
}

}  // namespace tv
