// fp32 tree-verification attention for gfx950 (head dimension 64 or 128, plain ALUs).
//
// This is the full-precision path: same masking rules as the bf16 MFMA kernel (Section 2 tree
// attention; Section 3.1 contemplate rows and soft-prompt visibility), every product and sum in
// fp32.  One workgroup owns 16 query rows of one query head and streams all keys of the sequence
// through LDS in tiles of 64; a wave owns 4 of the rows.  Scores: lane = key.  Values: lane = d.
#include <atomic>

#include "tv_internal.hpp"

namespace tv {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kRowsPerWave = 4;
constexpr int kRowsPerWg = kWaves * kRowsPerWave;
constexpr int kTile = 64;
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int D>
struct F32Smem {
    float k[kTile][D + 4];        // +4: rows stay 16-byte aligned and 16 lanes reading 16 bytes each at one d hit all banks
    float v[kTile][D];
    float q[kRowsPerWg][D];
    float p[kWaves][kRowsPerWave][kTile];
    int parent[kMaxRows];
    unsigned char kind[kMaxRows];
    int flag;
};

template <int D>
__global__ __launch_bounds__(kThreads) void attn_f32_kernel(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    F32Smem<D>& sm = *reinterpret_cast<F32Smem<D>*>(smem_raw);
    const int rb = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int M = a.M, g = h / a.G;
    constexpr int DPL = D / kWave;          // output columns per lane
    constexpr int kQPer = kRowsPerWg * D / 4 / kThreads;      // 16-byte pieces of the query block per thread
    constexpr int kTilePer = kTile * D / 4 / kThreads;        // ... of a K (or V) tile per thread

    // everything that does not hang on the prefix length is requested at once: the two per-sequence scalars, the
    // tree, the query block (into registers)
    const int P = a.prefix_len[b];
    const int64_t kv_first = a.kv_offset[b];
    const float* q = static_cast<const float*>(a.q);
    float* out = static_cast<float*>(a.out);
    const int row0 = rb * kRowsPerWg;
    int r_parent = 0;
    unsigned char r_kind = 0;
    if (tid < M) {                           // (M <= kMaxRows < kThreads)
        r_parent = a.parent[(int64_t)b * M + tid];
        r_kind = a.kind[(int64_t)b * M + tid];
    }
    f32x4 r_q[kQPer];
#pragma unroll
    for (int k = 0; k < kQPer; ++k) {
        const int idx = tid + k * kThreads, qi = idx / (D / 4), c4 = idx % (D / 4);
        const int i = min(row0 + qi, M - 1);
        r_q[k] = *reinterpret_cast<const f32x4*>(q + (((int64_t)b * M + i) * a.Hq + h) * D + c4 * 4);
    }
    if (tid < M) {
        sm.parent[tid] = r_parent;
        sm.kind[tid] = r_kind;
    }
#pragma unroll
    for (int k = 0; k < kQPer; ++k) {
        const int idx = tid + k * kThreads, qi = idx / (D / 4), c4 = idx % (D / 4);
        *reinterpret_cast<f32x4*>(&sm.q[qi][c4 * 4]) = r_q[k];
    }
    __syncthreads();
    int bad = validate_tree(sm.parent, sm.kind, M, &sm.flag);
    if (P < a.soft_len || P < 0 || P > a.max_prefix_len) bad |= TV_STATUS_BAD_PREFIX;
    if (rb == 0 && h == 0 && tid == 0) a.status[b] = bad;
    if (bad) {
        for (int idx = tid; idx < kRowsPerWg * D; idx += kThreads) {
            const int i = row0 + idx / D;
            if (i < M) out[(((int64_t)b * M + i) * a.Hq + h) * D + idx % D] = 0.f;
        }
        if (a.lse && tid < kRowsPerWg && row0 + tid < M) a.lse[((int64_t)b * a.Hq + h) * M + row0 + tid] = 0.f;
        return;
    }

    const int Lk = P + M;
    const float* kb = static_cast<const float*>(a.k) + kv_first * a.tok_stride + (int64_t)g * a.head_stride;
    const float* vb = static_cast<const float*>(a.v) + kv_first * a.tok_stride + (int64_t)g * a.head_stride;
    // a tile's 16-byte pieces, held in registers between their request and the moment the LDS tile is free
    f32x4 r_k[kTilePer], r_v[kTilePer];
#define TV_REQUEST_TILE(T0)                                                                            \
    _Pragma("unroll") for (int k = 0; k < kTilePer; ++k) {                                             \
        const int idx = tid + k * kThreads, key = idx / (D / 4), c4 = idx % (D / 4);                   \
        const int64_t src = (int64_t)min((T0) + key, Lk - 1) * a.tok_stride + c4 * 4;                  \
        r_k[k] = *reinterpret_cast<const f32x4*>(kb + src);                                           \
        r_v[k] = *reinterpret_cast<const f32x4*>(vb + src);                                           \
    }
    TV_REQUEST_TILE(0)

    // per-row state of this wave's rows (wave-uniform values live in every lane)
    int row[kRowsPerWave];
    bool is_con[kRowsPerWave];
    unsigned long long bits0[kRowsPerWave], bits1[kRowsPerWave];
    float m[kRowsPerWave], l[kRowsPerWave], o[kRowsPerWave][DPL];
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        row[r] = min(row0 + wave * kRowsPerWave + r, M - 1);
        is_con[r] = (sm.kind[row[r]] == TV_KIND_CONTEMPLATE);
        ancestor_bits(sm.parent, row[r], &bits0[r], &bits1[r]);
        m[r] = -INFINITY;
        l[r] = 0.f;
#pragma unroll
        for (int c = 0; c < DPL; ++c) o[r][c] = 0.f;
    }

    for (int t0 = 0; t0 < Lk; t0 += kTile) {
        __syncthreads();       // previous tile fully consumed
#pragma unroll
        for (int k = 0; k < kTilePer; ++k) {
            const int idx = tid + k * kThreads, key = idx / (D / 4), c4 = idx % (D / 4);
            *reinterpret_cast<f32x4*>(&sm.k[key][c4 * 4]) = r_k[k];
            *reinterpret_cast<f32x4*>(&sm.v[key][c4 * 4]) = r_v[k];
        }
        if (t0 + kTile < Lk) {                                // the next tile travels while this one is worked on
            TV_REQUEST_TILE(t0 + kTile)
        }
        __syncthreads();

        // scores: lane = key; the key's row and the four query rows are read 16 bytes at a time
        const int kg = t0 + lane;          // this lane's key
        float sc[kRowsPerWave];
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) sc[r] = 0.f;
#pragma unroll 4
        for (int d = 0; d < D; d += 4) {
            const float4 kk = *reinterpret_cast<const float4*>(&sm.k[lane][d]);
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                const float4 qq = *reinterpret_cast<const float4*>(&sm.q[wave * kRowsPerWave + r][d]);
                // (one chain per row, d ascending: the order of the plain loop)
                sc[r] = fmaf(qq.x, kk.x, sc[r]);
                sc[r] = fmaf(qq.y, kk.y, sc[r]);
                sc[r] = fmaf(qq.z, kk.z, sc[r]);
                sc[r] = fmaf(qq.w, kk.w, sc[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            float s = sc[r] * a.scale;
            bool vis;
            if (kg < P) vis = (kg >= a.soft_len) || is_con[r];
            else if (kg < Lk) {
                const int j = kg - P;
                vis = ((j < 64 ? (bits0[r] >> j) : (bits1[r] >> (j - 64))) & 1ull) != 0;
            } else vis = false;
            s = vis ? s : -INFINITY;
            const float m_new = fmaxf(m[r], wave_max(s));
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = expf(m[r] - m_safe);          // 0 while nothing was visible yet
            const float p = expf(s - m_safe);                 // 0 for masked keys
            l[r] = l[r] * alpha + wave_sum(p);
            m[r] = m_new;
#pragma unroll
            for (int c = 0; c < DPL; ++c) o[r][c] *= alpha;
            sm.p[wave][r][lane] = p;
        }
        // same wave wrote and reads sm.p: LDS operations of one wave complete in order
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // values: lane = output column; four keys' weights per read, keys ascending
        for (int key = 0; key < kTile; key += 4) {
            float4 pw[kRowsPerWave];
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) pw[r] = *reinterpret_cast<const float4*>(&sm.p[wave][r][key]);
#pragma unroll
            for (int c = 0; c < DPL; ++c) {
                const float v0 = sm.v[key][c * kWave + lane], v1 = sm.v[key + 1][c * kWave + lane];
                const float v2 = sm.v[key + 2][c * kWave + lane], v3 = sm.v[key + 3][c * kWave + lane];
#pragma unroll
                for (int r = 0; r < kRowsPerWave; ++r) {
                    o[r][c] = fmaf(pw[r].x, v0, o[r][c]);
                    o[r][c] = fmaf(pw[r].y, v1, o[r][c]);
                    o[r][c] = fmaf(pw[r].z, v2, o[r][c]);
                    o[r][c] = fmaf(pw[r].w, v3, o[r][c]);
                }
            }
        }
    }

#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        const int i = row0 + wave * kRowsPerWave + r;
        if (i >= M) continue;
        const float inv = 1.f / l[r];
#pragma unroll
        for (int c = 0; c < DPL; ++c)
            out[(((int64_t)b * M + i) * a.Hq + h) * D + c * kWave + lane] = o[r][c] * inv;
        if (a.lse && lane == 0) a.lse[((int64_t)b * a.Hq + h) * M + i] = m[r] + logf(l[r]);
    }
}

#undef TV_REQUEST_TILE

template <int D>
hipError_t launch_f32(const AttnArgs& a, hipStream_t s) {
    static std::atomic<unsigned> attr_done{0};       // one bit per device
    const size_t smem = sizeof(F32Smem<D>);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned bit = 1u << (dev & 31);
    if (!(attr_done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_f32_kernel<D>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_release);
    }
    const dim3 grid((a.M + kRowsPerWg - 1) / kRowsPerWg, a.Hq, a.B);
    attn_f32_kernel<D><<<grid, kThreads, smem, s>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention_f32(const AttnArgs& a, hipStream_t s) {
    if (a.D == 64) return launch_f32<64>(a, s);
    return launch_f32<128>(a, s);
}

}  // namespace tv
