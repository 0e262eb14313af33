// bf16 tree-verification attention for gfx950 (head dimension 128): MFMA 32x32x16 with fp32
// accumulation, online softmax, split over the keys with a second small combine kernel.
//
// What is computed: Section 2 (tree attention over the draft tree) and Section 3.1 (contemplate
// rows as extra tree rows; only they may attend to the soft-prompt slots) of the paper.
//
// Mapping
//   - The G = Hq/Hkv query heads of one KV head times the M rows are packed into G*M rows
//     r = head_in_group*M + row; a workgroup owns 64 consecutive packed rows of one KV head and
//     one of n_chunks ranges of the sequence's keys.  All four waves work on the same 64 rows;
//     the keys of the range are dealt to the waves in contiguous runs of 32-key tiles, so K and V
//     are read from HBM once per row block and each wave streams its own tiles through its own
//     LDS buffers (no workgroup barrier inside the loop).  The four waves' (max, sum, O) are
//     merged through LDS at the end.
//   - Scores are formed transposed, S^T = K Q^T: A = K tile (keys x d) read from LDS, B = Q^T held
//     in registers for the whole kernel.  In the 32x32 accumulator a lane then holds one query
//     (column) and 16 keys (rows), which is exactly the B-operand layout of O^T += V^T P^T, so the
//     probabilities never leave registers; V^T is read with the LDS transpose load.  The softmax
//     row reductions are in-lane plus one exchange between the wave's halves.
//   - The mask touches only tiles that overlap the soft-prompt slots or the new rows; all other
//     tiles run mask-free.  The ancestor mask is two 64-bit words per row, built in the prologue
//     from the parent array.
#include <atomic>

#include "tv_internal.hpp"

namespace tv {

namespace {

// memory is reinterpreted between these vector types (global <-> LDS <-> MFMA operands)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8), may_alias));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4), may_alias));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4), may_alias));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4), may_alias));

constexpr int kD = 128;
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kQRows = 64;                 // packed query rows per workgroup
constexpr int kTK = 32;                    // keys per tile
constexpr int kKStride = 272;              // bytes per K row in LDS (256 + 16: conflict-free 16-byte reads down a column of keys)
constexpr int kVStride = 288;              // bytes per V row in LDS (256 + 32: conflict-free transposed 8-byte reads)
constexpr int kKTile = kTK * kKStride;
constexpr int kVTile = kTK * kVStride;
constexpr int kStages = 2;
constexpr int kWaveLds = kStages * (kKTile + kVTile);      // 35840
constexpr int kOStride = kD + 4;           // floats per row of the merge buffer
constexpr int kMergeBytes = kWaves * kQRows * kOStride * 4;   // 135168
constexpr int kStreamBytes = kWaves * kWaveLds;              // 143360
constexpr int kBigBytes = kStreamBytes > kMergeBytes ? kStreamBytes : kMergeBytes;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kTau = 8.f;                // the running max is only raised when it lags by more than 2^kTau

struct Bf16Smem {
    unsigned char big[kBigBytes];          // per-wave K/V stages, later the merge buffer
    float ml[kWaves][kQRows][2];
    int parent[kMaxRows];
    unsigned char kind[kMaxRows];
    int flag;
};

__device__ __forceinline__ float cross_half_max(float x) {
    // lanes l and l^32 exchange: result0 = [x.lo, x.lo], result1 = [x.hi, x.hi]
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float cross_half_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ __launch_bounds__(kThreads, 1) void attn_bf16_kernel(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Bf16Smem& sm = *reinterpret_cast<Bf16Smem*>(smem_raw);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int ln = lane & 31, hf = lane >> 5;
    // blockIdx.x = g + Hkv * (rb + row_blocks * chunk): consecutive workgroups (hence the XCDs they are
    // dealt to round-robin) differ in KV head first, so each XCD's L2 sees few heads
    int bx = blockIdx.x;
    const int g = bx % a.Hkv; bx /= a.Hkv;
    const int rb = bx % a.row_blocks;
    const int chunk = bx / a.row_blocks;
    const int b = blockIdx.y;
    const int M = a.M, G = a.G;

    for (int i = tid; i < M; i += kThreads) {
        sm.parent[i] = a.parent[(int64_t)b * M + i];
        sm.kind[i] = a.kind[(int64_t)b * M + i];
    }
    __syncthreads();
    int bad = validate_tree(sm.parent, sm.kind, M, &sm.flag);
    const int P = a.prefix_len[b];
    if (P < a.soft_len || P < 0 || P > a.max_prefix_len) bad |= TV_STATUS_BAD_PREFIX;
    if (blockIdx.x == 0 && tid == 0) a.status[b] = bad;
    const int n_rows = G * M;
    unsigned short* out16 = static_cast<unsigned short*>(a.out);
    if (bad) {
        if (a.n_chunks == 1) {       // otherwise the combine kernel writes the zeros
            for (int idx = tid; idx < kQRows * kD; idx += kThreads) {
                const int r = rb * kQRows + idx / kD;
                if (r < n_rows)
                    out16[(((int64_t)b * M + r % M) * a.Hq + g * G + r / M) * kD + idx % kD] = 0;
            }
            if (a.lse && tid < kQRows && rb * kQRows + tid < n_rows) {
                const int r = rb * kQRows + tid;
                a.lse[((int64_t)b * a.Hq + g * G + r / M) * M + r % M] = 0.f;
            }
        }
        return;
    }

    // ---- this lane's two queries (column ln of query block 0 and 1) --------------------------------
    bf16x8 qreg[2][8];
    bool is_con[2];
    unsigned long long bits0[2], bits1[2];
    const unsigned short* q16 = static_cast<const unsigned short*>(a.q);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int r = min(rb * kQRows + qb * 32 + ln, n_rows - 1);
        const int i = r % M, h = g * G + r / M;
        const unsigned short* qp = q16 + (((int64_t)b * M + i) * a.Hq + h) * kD + hf * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
        is_con[qb] = (sm.kind[i] == TV_KIND_CONTEMPLATE);
        ancestor_bits(sm.parent, i, &bits0[qb], &bits1[qb]);
    }

    // ---- this wave's run of tiles -----------------------------------------------------------------------
    const int Lk = P + M;
    const int n_tiles = (Lk + kTK - 1) / kTK;
    const int n_slots = a.n_chunks * kWaves;
    const int slot = chunk * kWaves + wave;
    const int t_begin = (int)((int64_t)slot * n_tiles / n_slots);
    const int t_end = (int)((int64_t)(slot + 1) * n_tiles / n_slots);

    const int64_t tok_bytes = a.tok_stride * 2;
    const unsigned char* kbase = static_cast<const unsigned char*>(a.k) + (a.kv_offset[b] * a.tok_stride + (int64_t)g * a.head_stride) * 2;
    const unsigned char* vbase = static_cast<const unsigned char*>(a.v) + (a.kv_offset[b] * a.tok_stride + (int64_t)g * a.head_stride) * 2;
    unsigned char* my_lds = sm.big + wave * kWaveLds;

    const float c = a.scale * kLog2e;
    float m_run[2] = {-INFINITY, -INFINITY};    // running max, in log2 units (score * c)
    float l_run[2] = {0.f, 0.f};                // this lane's share of the running sum
    f32x16 o[4][2];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[dt][qb][j] = 0.f;

    u32x4 kst[8], vst[8];      // one tile in flight from HBM
    const int ld_row = lane >> 4, ld_seg = lane & 15;
    auto issue_loads = [&](int t) {
        const int k0 = t * kTK;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int key = min(k0 + 4 * j + ld_row, Lk - 1);      // never read past the sequence's rows
            const int64_t off = (int64_t)key * tok_bytes + ld_seg * 16;
            kst[j] = *reinterpret_cast<const u32x4*>(kbase + off);
            vst[j] = *reinterpret_cast<const u32x4*>(vbase + off);
        }
    };
    auto stash = [&](int stage) {
        unsigned char* kd = my_lds + stage * (kKTile + kVTile);
        unsigned char* vd = kd + kKTile;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            *reinterpret_cast<u32x4*>(kd + (4 * j + ld_row) * kKStride + ld_seg * 16) = kst[j];
            *reinterpret_cast<u32x4*>(vd + (4 * j + ld_row) * kVStride + ld_seg * 16) = vst[j];
        }
    };

    if (t_begin < t_end) {
        issue_loads(t_begin);
        stash(0);
    }
    for (int t = t_begin; t < t_end; ++t) {
        const int stage = (t - t_begin) & 1;
        if (t + 1 < t_end) issue_loads(t + 1);
        // one wave writes and reads its own buffers; LDS operations of a wave complete in order
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const unsigned char* kt = my_lds + stage * (kKTile + kVTile);
        const unsigned char* vt = kt + kKTile;
        const int k0 = t * kTK;

        // S^T = K Q^T
        f32x16 s[2];
#pragma unroll
        for (int j = 0; j < 16; ++j) { s[0][j] = 0.f; s[1][j] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 ka = *reinterpret_cast<const bf16x8*>(kt + ln * kKStride + ks * 32 + hf * 16);
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[0][ks], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[1][ks], s[1], 0, 0, 0);
        }

        // mask (only tiles touching the soft-prompt slots, the new rows or the tail)
        const bool need_mask = (k0 < a.soft_len) || (k0 + kTK > P);
        if (need_mask) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int kg = k0 + 8 * (j >> 2) + 4 * hf + (j & 3);
                    bool vis;
                    if (kg < P) vis = (kg >= a.soft_len) || is_con[qb];
                    else if (kg < Lk) {
                        const int jj = kg - P;
                        vis = ((jj < 64 ? (bits0[qb] >> jj) : (bits1[qb] >> (jj - 64))) & 1ull) != 0;
                    } else vis = false;
                    s[qb][j] = vis ? s[qb][j] : -INFINITY;
                }
        }

        // online softmax; the max is raised lazily (probabilities may reach 2^kTau, harmless in fp32/bf16)
        float tmax[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float x = s[qb][0];
#pragma unroll
            for (int j = 1; j < 16; ++j) x = fmaxf(x, s[qb][j]);
            tmax[qb] = cross_half_max(x) * c;
        }
        const bool raise0 = tmax[0] > m_run[0] + kTau, raise1 = tmax[1] > m_run[1] + kTau;
        if (__any(raise0 || raise1)) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const bool raise = qb ? raise1 : raise0;
                const float m_new = raise ? tmax[qb] : m_run[qb];
                const float alpha = raise ? __builtin_amdgcn_exp2f(m_run[qb] - m_new) : 1.f;   // exp2(-inf) = 0
                m_run[qb] = m_new;
                l_run[qb] *= alpha;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int j = 0; j < 16; ++j) o[dt][qb][j] *= alpha;
            }
        }
        bf16x8 pb[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float mc = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[qb][j], c, -mc));
                sum += p;
                pb[qb][j >> 3][j & 7] = (__bf16)p;
            }
            l_run[qb] += sum;
        }

        // O^T += V^T P^T
        const int g16 = lane >> 4, i16 = lane & 15;
        const unsigned char* vrow = vt + (4 * (g16 >> 1) + (i16 >> 2)) * kVStride + ((g16 & 1) * 16 + (i16 & 3) * 4) * 2;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const unsigned char* p0 = vrow + (16 * ks) * kVStride + dt * 64;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (bf16x4 __attribute__((address_space(3)))*)(p0));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (bf16x4 __attribute__((address_space(3)))*)(p0 + 8 * kVStride));
                bf16x8 va;
                va[0] = lo[0]; va[1] = lo[1]; va[2] = lo[2]; va[3] = lo[3];
                va[4] = hi[0]; va[5] = hi[1]; va[6] = hi[2]; va[7] = hi[3];
                o[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[0][ks], o[dt][0], 0, 0, 0);
                o[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[1][ks], o[dt][1], 0, 0, 0);
            }
        }
        if (t + 1 < t_end) stash(stage ^ 1);
    }

    // ---- merge the four waves through LDS -------------------------------------------------------------
    __syncthreads();       // every wave is done with its stage buffers
    float* mbuf = reinterpret_cast<float*>(sm.big);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = cross_half_sum(l_run[qb]);
        if (hf == 0) {
            sm.ml[wave][qb * 32 + ln][0] = m_run[qb];
            sm.ml[wave][qb * 32 + ln][1] = l_tot;
        }
        float* orow = mbuf + ((wave * kQRows) + qb * 32 + ln) * kOStride;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int jg = 0; jg < 4; ++jg) {
                f32x4 x = {o[dt][qb][4 * jg], o[dt][qb][4 * jg + 1], o[dt][qb][4 * jg + 2], o[dt][qb][4 * jg + 3]};
                *reinterpret_cast<f32x4*>(orow + dt * 32 + 8 * jg + 4 * hf) = x;
            }
    }
    __syncthreads();
    {
        const int qi = tid >> 2, dq = tid & 3;       // query row of the block, 32-wide column slice
        float mw[kWaves], mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { mw[w] = sm.ml[w][qi][0]; mx = fmaxf(mx, mw[w]); }
        const float mxs = (mx == -INFINITY) ? 0.f : mx;
        float wgt[kWaves], L = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            wgt[w] = __builtin_amdgcn_exp2f(mw[w] - mxs);
            L += wgt[w] * sm.ml[w][qi][1];
        }
        const int r = rb * kQRows + qi;
        const bool live = r < n_rows;
        const int i = live ? r % M : 0, h = g * G + (live ? r / M : 0);
        if (a.n_chunks == 1) {
            const float inv = 1.f / L;
            unsigned short* dst = out16 + (((int64_t)b * M + i) * a.Hq + h) * kD + dq * 32;
#pragma unroll
            for (int e = 0; e < 32; e += 4) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const f32x4 x = *reinterpret_cast<const f32x4*>(mbuf + (w * kQRows + qi) * kOStride + dq * 32 + e);
                    acc += x * wgt[w];
                }
                bf16x4 ob;
                ob[0] = (__bf16)(acc[0] * inv); ob[1] = (__bf16)(acc[1] * inv);
                ob[2] = (__bf16)(acc[2] * inv); ob[3] = (__bf16)(acc[3] * inv);
                if (live) *reinterpret_cast<bf16x4*>(dst + e) = ob;
            }
            if (a.lse && live && dq == 0) a.lse[((int64_t)b * a.Hq + h) * M + i] = (mx + log2f(L)) * kLn2;
        } else {
            const int64_t blk = (((int64_t)b * a.n_chunks + chunk) * a.Hkv + g) * a.row_blocks + rb;
            float* dst = a.part_o + (blk * kQRows + qi) * kD + dq * 32;
#pragma unroll
            for (int e = 0; e < 32; e += 4) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const f32x4 x = *reinterpret_cast<const f32x4*>(mbuf + (w * kQRows + qi) * kOStride + dq * 32 + e);
                    acc += x * wgt[w];
                }
                *reinterpret_cast<f32x4*>(dst + e) = acc;
            }
            if (dq == 0) {
                a.part_ml[(blk * kQRows + qi) * 2 + 0] = mx;
                a.part_ml[(blk * kQRows + qi) * 2 + 1] = L;
            }
        }
    }
}

// Merges the n_chunks partial results of every output row.  32 threads per row (4 columns each).
__global__ __launch_bounds__(256) void attn_bf16_combine_kernel(AttnArgs a) {
    const int rows_per_wg = 256 / 32;
    const int64_t row = (int64_t)blockIdx.x * rows_per_wg + threadIdx.x / 32;     // over B*M*Hq
    const int64_t total = (int64_t)a.B * a.M * a.Hq;
    if (row >= total) return;
    const int h = (int)(row % a.Hq);
    const int i = (int)((row / a.Hq) % a.M);
    const int b = (int)(row / ((int64_t)a.Hq * a.M));
    const int d0 = (threadIdx.x % 32) * 4;
    unsigned short* dst = static_cast<unsigned short*>(a.out) + row * kD + d0;
    if (a.status[b] != 0) {
        *reinterpret_cast<uint2*>(dst) = make_uint2(0u, 0u);
        if (a.lse && d0 == 0) a.lse[((int64_t)b * a.Hq + h) * a.M + i] = 0.f;
        return;
    }
    const int g = h / a.G, r = (h % a.G) * a.M + i;
    const int rb = r / kQRows, qi = r % kQRows;
    float mx = -INFINITY;
    for (int ch = 0; ch < a.n_chunks; ++ch) {
        const int64_t blk = (((int64_t)b * a.n_chunks + ch) * a.Hkv + g) * a.row_blocks + rb;
        mx = fmaxf(mx, a.part_ml[(blk * kQRows + qi) * 2]);
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float L = 0.f;
    for (int ch = 0; ch < a.n_chunks; ++ch) {
        const int64_t blk = (((int64_t)b * a.n_chunks + ch) * a.Hkv + g) * a.row_blocks + rb;
        const float w = __builtin_amdgcn_exp2f(a.part_ml[(blk * kQRows + qi) * 2] - mx);
        L += w * a.part_ml[(blk * kQRows + qi) * 2 + 1];
        acc += *reinterpret_cast<const f32x4*>(a.part_o + (blk * kQRows + qi) * kD + d0) * w;
    }
    const float inv = 1.f / L;
    bf16x4 ob;
    ob[0] = (__bf16)(acc[0] * inv); ob[1] = (__bf16)(acc[1] * inv);
    ob[2] = (__bf16)(acc[2] * inv); ob[3] = (__bf16)(acc[3] * inv);
    *reinterpret_cast<bf16x4*>(dst) = ob;
    if (a.lse && d0 == 0) a.lse[((int64_t)b * a.Hq + h) * a.M + i] = (mx + log2f(L)) * kLn2;
}

}  // namespace

hipError_t launch_attention_bf16(const AttnArgs& a, hipStream_t s) {
    static std::atomic<unsigned> attr_done{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned bit = 1u << (dev & 31);
    if (!(attr_done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Bf16Smem));
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_release);
    }
    const dim3 grid(a.Hkv * a.row_blocks * a.n_chunks, a.B);
    attn_bf16_kernel<<<grid, kThreads, sizeof(Bf16Smem), s>>>(a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.n_chunks > 1) {
        const int64_t rows = (int64_t)a.B * a.M * a.Hq;
        attn_bf16_combine_kernel<<<dim3((unsigned)((rows + 7) / 8)), 256, 0, s>>>(a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace tv
