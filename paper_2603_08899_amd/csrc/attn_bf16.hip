// bf16 tree-verification attention for gfx950 (head dimension 128): MFMA 32x32x16 with fp32
// accumulation, online softmax, keys split over workgroups with a small combine kernel.
//
// What is computed: Section 2 (tree attention over the draft tree) and Section 3.1 (contemplate
// rows as extra tree rows; only they may attend to the soft-prompt slots) of the paper.
//
// Mapping
//   - The G = Hq/Hkv query heads of one KV head times the M rows are packed into G*M rows
//     r = head_in_group*M + row.  A wave owns 32 consecutive packed rows: Q^T for its rows stays in
//     registers as the MFMA B operand for the whole kernel.
//   - A workgroup (8 waves, two per SIMD) covers RB*64 packed rows and one of n_chunks ranges of the
//     sequence's keys.  Its waves form NS = 4/RB key streams: the range is cut into NS contiguous runs of
//     32-key tiles, and the 2*RB waves of a stream - one per 32-row slice - consume the same K/V tiles from LDS.
//   - K/V tiles and the Q block go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no registers),
//     tiles ahead of their use into a ring of 2*RB stages per stream.  Rows are 256 bytes; bank conflicts are
//     avoided by an XOR swizzle of the 16-byte segments which is applied on the global-address side.
//   - Scores are formed transposed, S^T = K Q^T (A = K tile from LDS).  In the 32x32 accumulator a
//     lane then holds one query (column) and 16 keys (rows): exactly the B-operand layout of
//     O^T += V^T P^T, so probabilities stay in registers; V^T comes from the LDS transpose load.
//     Softmax row reductions are in-lane plus one exchange between the wave's halves.
//   - Only tiles overlapping the soft-prompt slots, the new rows or the tail are masked, with a
//     32-bit visibility word per (lane, query) derived from the two-word ancestor mask.
//   - RB = 1 (64-row workgroups, four streams of two stages: the smallest partial results, for short and
//     medium contexts): one barrier per tile; the product O^T += V^T P^T of a tile is issued one tile late,
//     next to the following tile's exponentials.
//     RB = 2, 4 (128- and 256-row workgroups, stages enough to keep tiles several rounds ahead, for long
//     contexts and batches): a tile takes two barrier slots, scores in one, softmax and O^T product in the
//     next, and the two waves of a SIMD are one slot apart.
//   - Several sequences are served longest prefix first (the second grid index is a length rank), so that the
//     long runs of tiles start early and the short ones fill in behind them.
//   - Streams are merged through LDS; with n_chunks > 1 partial results (O / L in bf16, max and L in fp32)
//     go to the workspace and attn_bf16_combine_kernel finishes.
#include <atomic>

#include "attn_bf16_common.hpp"

namespace tv {

namespace {

// RB: 64-row blocks covered by one workgroup (1, 2 or 4)
// The two per-sequence arrays and the sequence count come as arguments of their own, ahead of the rest: the first
// tile's address hangs on them, and leading scalar arguments are in registers when a wave starts (kernel-argument preload, see the
// build flags), which takes one scalar-load latency off the start of every workgroup.
template <int RB>
__global__ __launch_bounds__(512, 1) void attn_bf16_kernel(const int32_t* prefix_len, const int64_t* kv_offset,
                                                           int n_seq, AttnArgs a) {
    constexpr int NW = 8;                              // waves per workgroup, two per SIMD (waves w and w+4)
    constexpr int kThreads = NW * kWave;
    constexpr int WROWS = 32;                          // packed rows per wave
    constexpr int WPS = (kQRows * RB) / WROWS;         // waves per key stream (one per row slice)
    constexpr int NS = NW / WPS;                       // key streams per workgroup
    constexpr int S = kRingBytes / (NS * kStageBytes); // stages per stream: 2, 4 or 8 (= 2*RB)
    constexpr int PER = 16 / WPS;                      // direct-to-LDS loads per tile per wave
    static_assert(S == 2 * RB && PER >= 2, "stage ring layout");
    extern __shared__ __align__(1024) unsigned char smem_raw[];   // stage bases are multiples of 256 (see k_base)
    Bf16Smem& sm = *reinterpret_cast<Bf16Smem*>(smem_raw);
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int ln = lane & 31, hf = lane >> 5;
    const int wsub = wave % WPS, st = wave / WPS;      // row slice and key stream of this wave
    // blockIdx.x = g + Hkv * (rbg + row_groups * chunk): neighbouring workgroups (dealt round-robin to
    // the XCDs) differ in KV head first, so one XCD's L2 serves few heads
    int bx = blockIdx.x;
    const int g = bx % a.Hkv; bx /= a.Hkv;
    const int row_groups = a.row_blocks / RB;
    const int rbg = bx % row_groups;
    const int chunk = bx / row_groups;
    const int row0 = rbg * RB * kQRows + wsub * WROWS; // this wave's first packed row
    int b = blockIdx.y;                                // replaced by a length rank below when there are several
    const int M = a.M, G = a.G;
    const int n_rows = G * M;
    unsigned char* ring = sm.big + st * (S * kStageBytes);
    const unsigned ring_addr = lds_address(ring);
    const int l_row = lane >> 4, l_seg = lane & 15;    // a direct-to-LDS load lands lane l at row l/16, segment l%16

    // The two per-sequence scalars everything below waits for are requested first, so that their latency runs
    // under the Q requests (the assembly statements of those keep later loads from moving up past them).
    int P;
    int64_t kv_first_row;
    if (n_seq > 1 && n_seq <= kWave) {
        // Several sequences: the second grid index counts them by decreasing prefix length (ties by index), so
        // the workgroups of the longest come first in the dispatch order and the short ones fill in behind
        // them.  Every wave ranks the sequences for itself, lane l holding sequence l; the ranks are a
        // permutation of 0 .. n_seq-1 whatever the lengths are, so each sequence is still served exactly once.
        const bool live = lane < n_seq;
        const int len = live ? prefix_len[lane] : -1;
        const long long off = live ? kv_offset[lane] : 0;
        int rank = 0;
        for (int j = 0; j < n_seq; ++j) {
            const int len_j = __builtin_amdgcn_readlane(len, j);
            rank += (len_j > len || (len_j == len && j < lane)) ? 1 : 0;
        }
        b = __ffsll((long long)__ballot(live && rank == (int)blockIdx.y)) - 1;
        P = __builtin_amdgcn_readlane(len, b);
        const unsigned lo = __builtin_amdgcn_readlane((unsigned)off, b);
        const unsigned hi = __builtin_amdgcn_readlane((unsigned)(off >> 32), b);
        kv_first_row = (long long)(((unsigned long long)hi << 32) | lo);
    } else {
        P = prefix_len[b];
        kv_first_row = kv_offset[b];
    }

    // ---- tree rows (64-row workgroups): parent and kind - or, from a prepared tree, the ancestor masks, kinds and
    //      verdict - go straight into LDS, requested by wave 0 ahead of everything else, so that the wait for the
    //      query block below covers them and no register load makes the compiler wait for the tiles requested in
    //      between -----------------------------------------------------------------------------------------
    const PreparedTree* prep = a.prepared ? reinterpret_cast<const PreparedTree*>(a.prepared) + b : nullptr;
    if (RB == 1 && wave == 0) {
        if (prep) {
            const unsigned long long prep_base = scalar_base(prep);
            for (int j = 0; j < (M + kWave - 1) / kWave; ++j) {   // (the record holds kMaxRows rows, zeros past M)
                const unsigned row = (unsigned)(j * kWave + lane);
                dma16(lds_address(&sm.bits[j * kWave][0]), prep_base, (unsigned)offsetof(PreparedTree, bits) + row * 16u);
                dma1(lds_address(&sm.kind[j * kWave]), prep_base, (unsigned)offsetof(PreparedTree, kind) + row);
            }
            dma4(lds_address(&sm.prep_status[0]), prep_base, (unsigned)offsetof(PreparedTree, status));
        } else {
            const unsigned long long par_base = scalar_base(a.parent + (int64_t)b * M);
            const unsigned long long kind_base = scalar_base(a.kind + (int64_t)b * M);
            for (int j = 0; j < (M + kWave - 1) / kWave; ++j) {   // rows past M repeat row M-1 (never looked at)
                const unsigned row = (unsigned)min(j * kWave + lane, M - 1);
                dma4(lds_address(&sm.parent[j * kWave]), par_base, row * 4u);
                dma1(lds_address(&sm.kind[j * kWave]), kind_base, row);
            }
        }
    }

    // ---- Q for this wave's rows: HBM -> LDS -----------------------------------------------------------
    // A 32-row slice of the query block is laid out like a K tile, with the same segment swizzle.  64-row
    // workgroups keep the block (two slices) in its own area and every wave requests an eighth of it; the larger
    // shapes stage each stream's slices in the upper half of its ring, which is free at this point.
    const int q_off = (S / 2) * kStageBytes + wsub * kTileBytes;
    const unsigned q_slice_addr = (RB == 1) ? lds_address(smem_raw + kQAreaOffset) + wsub * kTileBytes
                                            : ring_addr + q_off;
    {
        const unsigned q_stage = __builtin_amdgcn_readfirstlane(q_slice_addr);
        const unsigned long long q_sbase =
            scalar_base(static_cast<const unsigned char*>(a.q) + (int64_t)b * M * a.Hq * (kD * 2));
        constexpr int kQLoads = (RB == 1) ? 2 : 8;
#pragma unroll
        for (int jj = 0; jj < kQLoads; ++jj) {
            const int j = (RB == 1) ? 2 * st + jj : jj;
            const int row = 4 * j + l_row;            // row inside the query block: selects the swizzle
            const int r = min(row0 + row, n_rows - 1);                 // padding rows re-read the last packed row
            const int hl = (int)(((float)r + 0.5f) * a.inv_M);         // r / M (exact for these sizes)
            const int i = r - hl * M;                                  // (head in group, tree row) of packed row r
            const unsigned off = (unsigned)((i * a.Hq + g * G + hl) * (kD * 2) + ((l_seg ^ (row & 15)) * 16));
            dma16(q_stage + j * 1024, q_sbase, off);
        }
    }

    // ---- key range, first K/V tiles (they depend on the prefix length only) ---------------------------
    const bool bad_prefix = (P < a.soft_len || P < 0 || P > a.max_prefix_len);
    const int Lk = bad_prefix ? M : P + M;
    const int n_tiles = (Lk + kTK - 1) / kTK;
    const int n_slots = a.n_chunks * NS;
    const int slot0 = chunk * NS;
    // slot u gets tiles_per_slot tiles, the first `extra` slots one more (one 32-bit division)
    const int tiles_per_slot = (int)((unsigned)n_tiles / (unsigned)n_slots);
    const int extra = n_tiles - tiles_per_slot * n_slots;
    const int slot = slot0 + st;
    const int t_begin = slot * tiles_per_slot + min(slot, extra);
    const int n_my = bad_prefix ? 0 : tiles_per_slot + (slot < extra ? 1 : 0);
    // the longest stream of the workgroup is its first one
    const int n_iter = bad_prefix ? 0 : tiles_per_slot + (slot0 < extra ? 1 : 0);
    auto tile_of = [&](int it) { return t_begin + it; };

    const int64_t seq_base = (kv_first_row * a.tok_stride + (int64_t)g * a.head_stride) * 2;
    const unsigned char* kbase = static_cast<const unsigned char*>(a.k) + seq_base;
    const unsigned char* vbase = static_cast<const unsigned char*>(a.v) + seq_base;
    const unsigned tok_bytes = (unsigned)(a.tok_stride * 2);

    // One tile: instruction j (0..7 K, 8..15 V) moves rows 4j..4j+3; lane l lands at byte 16*l of that 1 KB
    // block and fetches the logical segment that the swizzle stores there (K: segment ^ (row & 15); V: segment ^
    // 4 * (row & 3)).  This wave issues the instructions j = jj*WPS + wsub of each half.
    // What differs between the PER/2 request instructions of a half tile is kept per lane (the row block's offset
    // next to the lane's row and swizzled segment), so that one scalar base per half tile serves all of them and an
    // instruction costs a couple of scalar operations.
    constexpr int HP = PER / 2;                    // request instructions of this wave per half tile
    unsigned k_voff[HP], v_voff[HP];
#pragma unroll
    for (int jj = 0; jj < HP; ++jj) {
        const int jb = jj * WPS + wsub;            // 4-row block of the tile (0 .. 7)
        k_voff[jj] = (unsigned)(4 * jb + l_row) * tok_bytes + (unsigned)((l_seg ^ l_row ^ (4 * (jb & 3))) << 4);
        v_voff[jj] = (unsigned)(4 * jb + l_row) * tok_bytes + (unsigned)((l_seg ^ (l_row << 2)) << 4);
    }
    auto issue_half = [&](int t, int stage, int half) __attribute__((always_inline)) {      // half 0: K rows, half 1: V rows
        const int k0 = t * kTK;
        const unsigned dst = __builtin_amdgcn_readfirstlane(ring_addr + stage * kStageBytes + half * kTileBytes + wsub * 1024);
        const unsigned char* base = half ? vbase : kbase;
        if (k0 + kTK <= Lk) {
            const unsigned long long tile_base = scalar_base(base + (size_t)k0 * tok_bytes);
#pragma unroll
            for (int jj = 0; jj < HP; ++jj) dma16(dst + jj * (WPS * 1024), tile_base, half ? v_voff[jj] : k_voff[jj]);
        } else {                                             // last tile: never read past the sequence's rows
#pragma unroll
            for (int jj = 0; jj < HP; ++jj) {
                const int jb = jj * WPS + wsub;
                const int row = 4 * jb + l_row;
                const unsigned key = (unsigned)min(k0 + row, Lk - 1);
                const int seg = half ? (l_seg ^ (l_row << 2)) : (l_seg ^ (row & 15));
                dma16(dst + jj * (WPS * 1024), scalar_base(base), key * tok_bytes + (unsigned)(seg * 16));
            }
        }
    };
    auto issue_tile = [&](int t, int stage) { issue_half(t, stage, 0); issue_half(t, stage, 1); };
    // 64-row workgroups fill both stages of every stream here; the others the lower half of their rings
    constexpr int kFirstTiles = (RB == 1) ? S : S / 2;
#pragma unroll
    for (int i = 0; i < kFirstTiles; ++i)
        if (i < n_my) issue_tile(tile_of(i), i);

    // ---- tree, validation ------------------------------------------------------------------------------
    if (RB == 1) {
        // everything requested before the tiles (tree rows, query block) has landed once no more than the tile
        // requests are outstanding
        if (n_my >= 2) wait_vmcnt<2 * PER>();
        else if (n_my == 1) wait_vmcnt<PER>();
        else wait_vmcnt<0>();
    } else {
        // ordinary loads: the wait the compiler puts before the LDS writes also covers everything requested above
        if (tid < M) {
            if (prep) {
                sm.bits[tid][0] = prep->bits[tid][0];
                sm.bits[tid][1] = prep->bits[tid][1];
                sm.kind[tid] = prep->kind[tid];
            } else {
                sm.parent[tid] = a.parent[(int64_t)b * M + tid];
                sm.kind[tid] = a.kind[(int64_t)b * M + tid];
            }
        }
        if (prep && tid == 0) sm.prep_status[0] = prep->status;
        wait_vmcnt<0>();
    }
    if (tid == 0) sm.flag = 0;
    __syncthreads();
    // Row tid checks itself; a workgroup whose key range meets masked tiles (soft-prompt slots, new rows, the
    // tail) also walks the row's ancestors once and leaves the two mask words in LDS.  The walk only follows
    // parents that are smaller than the row they belong to, so it ends whatever the other rows hold.
    // With a prepared tree all of this was done once for the step: only the verdict is taken over.
    if (prep) {
        if (tid == 0) sm.flag = sm.prep_status[0];
    } else if (tid < M) {                                 // row tid (M <= 128 < kThreads)
        const int my_parent = sm.parent[tid], my_kind = sm.kind[tid] & 0xff;
        int bad = 0;
        if (my_parent < -1 || my_parent >= tid) bad |= TV_STATUS_BAD_PARENT;
        if (my_kind != TV_KIND_NODE && my_kind != TV_KIND_CONTEMPLATE) bad |= TV_STATUS_BAD_KIND;
        else if (my_parent >= 0 && my_parent < tid && my_kind == TV_KIND_NODE &&
                 (sm.kind[my_parent] & 0xff) == TV_KIND_CONTEMPLATE)
            bad |= TV_STATUS_BAD_KIND;
        const int wg_t_begin = slot0 * tiles_per_slot + min(slot0, extra);
        const int wg_t_end = (slot0 + NS) * tiles_per_slot + min(slot0 + NS, extra);
        if (wg_t_begin * kTK < a.soft_len || wg_t_end * kTK > P) {
            unsigned long long w0 = 0, w1 = 0;
            int j = tid;
            while (j >= 0) {
                if (j < 64) w0 |= 1ull << j; else w1 |= 1ull << (j - 64);
                const int pj = sm.parent[j];
                j = (pj < j) ? pj : -1;
            }
            sm.bits[tid][0] = w0;
            sm.bits[tid][1] = w1;
        }
        if (bad) atomicOr(&sm.flag, bad);     // looked at after the next barrier
    }

    // per-lane LDS offsets of the MFMA operands inside a tile
    // K (A operand of S^T): row ln, logical segment 2*ks + hf, stored at segment (2*ks + hf) ^ (ln & 15): the
    // offset for step ks is k_base ^ (ks << 5).  V^T (A operand of O^T): transposed 8-byte reads, 4 keys x 16 d
    // per 16 lanes; the offset for column block dt is v_base ^ (dt << 6).  Both XORs only touch bits 5..7, so
    // they commute with adding a stage base that is a multiple of 256.
    const unsigned k_base = (unsigned)(ln * kRowBytes + ((hf ^ (ln & 15)) << 4));
    unsigned v_base;
    {
        const int g16 = lane >> 4, i16 = lane & 15;
        const int row = 4 * (g16 >> 1) + (i16 >> 2);
        const int seg0 = 4 * (i16 >> 2) + (g16 & 1) * 2 + ((i16 & 3) >> 1);
        v_base = (unsigned)(kTileBytes + row * kRowBytes + seg0 * 16 + (i16 & 1) * 8);
    }
    typedef const bf16x8 __attribute__((address_space(3))) * lds_b128_ptr;
    typedef bf16x4 __attribute__((address_space(3))) * lds_b64_ptr;

    // ---- this lane's query (column ln of the query block): B operands of S^T, kept in registers ---------
    bf16x8 qreg[8];
    {
        const unsigned q_it = q_slice_addr + k_base;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[ks] = *(lds_b128_ptr)(q_it ^ (ks << 5));
    }
    const int tree_row = [&] {       // tree row of the query (the mask of a tile is derived from it on demand)
        const int r = min(row0 + ln, n_rows - 1);
        return r - (int)(((float)r + 0.5f) * a.inv_M) * M;             // r % M
    }();
    __syncthreads();         // the Q staging area goes back to the ring; every row's verdict is in sm.flag
    int bad = sm.flag;
    if (bad_prefix) bad |= TV_STATUS_BAD_PREFIX;
    if (blockIdx.x == 0 && tid == 0) a.status[b] = bad;
    unsigned short* out16 = static_cast<unsigned short*>(a.out);
    if (bad) {
        wait_vmcnt<0>();             // (tiles requested above land before the workgroup gives its LDS back)
        if (a.n_chunks == 1) {       // otherwise the combine kernel writes the zeros
            for (int idx = tid; idx < RB * kQRows * kD; idx += kThreads) {
                const int r = rbg * RB * kQRows + idx / kD;
                if (r < n_rows)
                    out16[(((int64_t)b * M + r % M) * a.Hq + g * G + r / M) * kD + idx % kD] = 0;
            }
            for (int idx = tid; idx < RB * kQRows; idx += kThreads) {
                const int r = rbg * RB * kQRows + idx;
                if (a.lse && r < n_rows) a.lse[((int64_t)b * a.Hq + g * G + r / M) * M + r % M] = 0.f;
            }
        }
        return;
    }

#pragma unroll
    for (int i = kFirstTiles; i < (RB == 1 ? S - 1 : S); ++i)       // (64-row workgroups have filled their ring)
        if (i < n_my) issue_tile(tile_of(i), i);

    const float c = a.scale * kLog2e;
    float m_run = -INFINITY, l_run = 0.f;       // running max in log2 units (score * c); this lane's share of the sum
    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[dt][j] = 0.f;

    // O^T += V^T P^T for one tile
    auto pv_mfma = [&](bf16x8 (&va)[8], bf16x8 (&pb)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ks * 4 + dt], pb[ks], o[dt], 0, 0, 0);
    };
    // K operands (A of S^T) of one tile: all eight reads are requested back to back
    auto read_k = [&](int it, bf16x8 (&ka)[8]) __attribute__((always_inline)) {
        const unsigned k_it = __builtin_amdgcn_readfirstlane(ring_addr + (it % S) * kStageBytes) + k_base;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) ka[ks] = *(lds_b128_ptr)(k_it ^ (ks << 5));
    };
    // V^T operands (A of O^T) of one tile
    auto read_v = [&](int it, bf16x8 (&va)[8]) __attribute__((always_inline)) {
        const unsigned v_it = __builtin_amdgcn_readfirstlane(ring_addr + (it % S) * kStageBytes) + v_base;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const unsigned p0 = (v_it ^ (dt << 6)) + ks * (16 * kRowBytes);
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(p0));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(p0 + 8 * kRowBytes));
                va[ks * 4 + dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };
    // S^T = K Q^T for one tile
    auto score_tile = [&](bf16x8 (&ka)[8], f32x16& s) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[ks], s, 0, 0, 0);
    };
    // Mask of a tile that touches the soft-prompt slots, the new rows or the tail (a few tiles per sequence):
    // from the row's ancestor mask, left in LDS by the prologue
    auto mask_tile = [&](int it, f32x16& s) __attribute__((always_inline)) {
        const int k0 = tile_of(it) * kTK;
        if ((k0 < a.soft_len) || (k0 + kTK > P)) {
            const unsigned long long bits0 = sm.bits[tree_row][0], bits1 = sm.bits[tree_row][1];
            const bool is_con = ((sm.kind[tree_row] & 0xff) == TV_KIND_CONTEMPLATE);
            const unsigned vis = tile_visibility(k0, P, a.soft_len, is_con, bits0, bits1) >> (4 * hf);
#pragma unroll
            for (int j = 0; j < 16; ++j) s[j] = (vis & (1u << (8 * (j >> 2) + (j & 3)))) ? s[j] : -INFINITY;
        }
    };
    // Largest score of the lane's query in the tile, in log2 units
    auto tile_max = [&](const f32x16& s) __attribute__((always_inline)) {
        float x = s[0];
#pragma unroll
        for (int j = 1; j < 16; ++j) x = fmaxf(x, s[j]);
        return cross_half_max(x) * c;
    };
    // The lane's query takes `tmax` as its new reference if that is what was asked for: O and the sum are rescaled
    auto rescale = [&](bool raise, float tmax) __attribute__((always_inline)) {
        const float m_new = raise ? tmax : m_run;
        const float alpha = raise ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;   // exp2(-inf) = 0
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[dt][j] *= alpha;
    };
    // Probabilities of the tile (relative to the running reference) as B operands of O^T, and their sum
    auto probabilities = [&](const f32x16& s, bf16x8 (&pb)[2]) __attribute__((always_inline)) {
        const float mc = (m_run == -INFINITY) ? 0.f : m_run;
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s[j], c, -mc));
            sum += p;
            pb[j >> 3][j & 7] = (__bf16)p;
        }
        l_run += sum;
    };
    // The running max is raised lazily: only when a tile's max exceeds it by more than 2^kTau (probabilities may
    // reach 2^kTau, harmless in fp32/bf16), so the rescale of O is rare.

    if (RB == 1) {
        // Four streams of two stages.  A tile takes two barrier slots: phase A = matrix work only - K operands, the
        // PREVIOUS tile's O^T += V^T P^T (its operands are in registers, so it runs while the K operands land) and
        // the score products; phase B = vector work only - the tile's V^T operands (requested first), mask, softmax.
        // The two waves of a SIMD (w and w+4, i.e. streams 0-1 and streams 2-3) are one phase apart:
        //   slot 2t   : waves 0-3 phase A of tile t,  waves 4-7 phase B of tile t-1
        //   slot 2t+1 : waves 0-3 phase B of tile t,  waves 4-7 phase A of tile t
        // With two stages a whole tile could only be requested one round ahead, so the halves of a stage are
        // refilled separately, each by the stream's own waves after the barrier that follows its last read: the K
        // half with K(t+2) at the end of phase B(t) (behind the vector work, when the request path is idle), the V
        // half with V(t+2) when the slot of phase A(t+1) opens - about a round and a half ahead of their use.  Requests of a wave, in
        // order: K0 V0 K1 V1 (prologue) | K2 | V2 | K3 | V3 ...  Both halves of the workgroup run their own copy
        // of the loop (2*n_iter+1 barriers each): with the phase order fixed the accumulators stay in place.
        bf16x8 va[8], pb[2];     // V^T operands and probabilities of the tile whose product is still to be issued
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int x = 0; x < 8; ++x) va[e][x] = (__bf16)0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int x = 0; x < 8; ++x) pb[ks][x] = (__bf16)0.f;
        f32x16 s;
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = 0.f;
        // opens the slot of phase A(t): K(t) has landed (younger requests: V(t), K(t+1)); V(t+1) may be requested
        auto open_a = [&](int t) __attribute__((always_inline)) {
            if (t < n_my) {
                if (t + 1 < n_my) {
                    if (t == 0) wait_vmcnt<3 * PER / 2>();      // (V0, K1 and V1 were all requested in the prologue)
                    else wait_vmcnt<PER>();
                } else {
                    wait_vmcnt<PER / 2>();
                }
            }
            __syncthreads();
            if (t >= 1 && t + 1 < n_my) issue_half(tile_of(t + 1), (t + 1) % S, 1);
        };
        // opens the slot of phase B(t): V(t) has landed (younger requests: K(t+1), V(t+1)); K(t+2) may be requested
        auto open_b = [&](int t) __attribute__((always_inline)) {
            if (t >= 0 && t < n_my) {
                if (t + 1 < n_my) wait_vmcnt<PER>();
                else wait_vmcnt<0>();
            }
            __syncthreads();
        };
        auto phase_a = [&](int t) __attribute__((always_inline)) {
            bf16x8 ka[8];        // all eight reads are requested first; the previous tile's product runs while they land
            read_k(t, ka);
            __builtin_amdgcn_sched_barrier(0);
            pv_mfma(va, pb);
            score_tile(ka, s);
        };
        auto phase_b = [&](int t) __attribute__((always_inline)) {
            read_v(t, va);                             // requested first: the LDS latency runs under the softmax
            __builtin_amdgcn_sched_barrier(0);
            mask_tile(t, s);
            const float tmax = tile_max(s);
            if (t == 0) m_run = tmax;                  // nothing accumulated yet: adopt the tile's max as the reference
            else if (__any(tmax > m_run + kTau)) rescale(tmax > m_run + kTau, tmax);      // rare
            probabilities(s, pb);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 2 < n_my) issue_half(tile_of(t + 2), t % S, 0);
        };
        if ((wave >> 2) == 0) {
            for (int t = 0; t < n_iter; ++t) {
                open_a(t);
                if (t < n_my) phase_a(t);
                open_b(t);
                if (t < n_my) phase_b(t);
            }
            __syncthreads();
        } else {
            for (int t = 0; t < n_iter; ++t) {
                open_b(t - 1);
                if (t >= 1 && t - 1 < n_my) phase_b(t - 1);
                open_a(t);
                if (t < n_my) phase_a(t);
            }
            open_b(n_iter - 1);
            if (n_iter >= 1 && n_iter - 1 < n_my) phase_b(n_iter - 1);       // (no tile at all: no trailing phase)
        }
        pv_mfma(va, pb);         // the last tile's product
    } else {
        // Waves that share one or two key streams (eight or four stages) take a tile in two phases, in two barrier
        // slots: phase A = K operands and the score products; phase B = V^T operands (requested first), mask,
        // softmax, then O^T += V^T P^T.  The two waves of a SIMD (w and w+4) are one phase apart, so that one's
        // matrix-heavy phase runs under the other's vector-heavy one; only the scores are carried between phases.
        //   slot 2t   : waves 0-3 phase A of tile t,  waves 4-7 phase B of tile t-1
        //   slot 2t+1 : waves 0-3 phase B of tile t,  waves 4-7 phase A of tile t
        // Every wave has waited for its part of tile t before the barrier that opens slot 2t.  The stage of tile t
        // is read for the last time in slot 2t+2 and refilled (tile t+S) after the barrier that opens slot 2t+3.
        // The two halves of the workgroup run separate copies of the loop (both meet 2*n_iter+1 barriers): with the
        // phase order fixed in each copy the accumulators stay in place.
        f32x16 s;
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = 0.f;
        // the barrier that opens slot 2t, once this wave's part of tile t has landed
        auto open_even = [&](int t) __attribute__((always_inline)) {
            if (t < n_my) {
                const int younger = min(n_my - 1, S - 1 + max(0, t - 1)) - t;       // tiles requested after tile t
                if (younger >= S - 1) wait_vmcnt<(S - 1) * PER>();
                else if (younger == S - 2) wait_vmcnt<(S - 2) * PER>();
                else wait_vmcnt<0>();
            }
            __syncthreads();
        };
        // the barrier that opens slot 2t+1; the stage of tile t-1 is free from here on
        auto open_odd = [&](int t) __attribute__((always_inline)) {
            __syncthreads();
            if (t >= 1 && t - 1 + S < n_my) issue_tile(tile_of(t - 1 + S), (t - 1) % S);
        };
        auto phase_a = [&](int t) __attribute__((always_inline)) {
            bf16x8 ka[8];
            read_k(t, ka);
            score_tile(ka, s);
        };
        auto phase_b = [&](int t) __attribute__((always_inline)) {
            bf16x8 va[8], pb[2];
            read_v(t, va);
            __builtin_amdgcn_sched_barrier(0);
            mask_tile(t, s);
            const float tmax = tile_max(s);
            if (t == 0) m_run = tmax;
            else if (__any(tmax > m_run + kTau)) rescale(tmax > m_run + kTau, tmax);      // rare
            probabilities(s, pb);
            pv_mfma(va, pb);
        };
        if ((wave >> 2) == 0) {
            for (int t = 0; t < n_iter; ++t) {
                open_even(t);
                if (t < n_my) phase_a(t);
                open_odd(t);
                if (t < n_my) phase_b(t);
            }
            open_even(n_iter);
        } else {
            for (int t = 0; t < n_iter; ++t) {
                open_even(t);
                if (t >= 1 && t - 1 < n_my) phase_b(t - 1);
                open_odd(t);
                if (t < n_my) phase_a(t);
            }
            open_even(n_iter);
            if (n_iter >= 1 && n_iter - 1 < n_my) phase_b(n_iter - 1);       // (no tile at all: no trailing phase)
        }
    }

    // ---- merge the streams through LDS -------------------------------------------------------------------
    // Merge buffer: [wave][its rows][32 float4]; float4 column c of a wave's row r is stored at column c ^ (r & 31).
    wait_vmcnt<0>();
    __syncthreads();       // every wave is done with the stage ring
    f32x4* mbuf = reinterpret_cast<f32x4*>(sm.big);
    {
        const float l_tot = cross_half_sum(l_run);
        const int mrow = wave * WROWS + ln;
        if (hf == 0) {
            sm.ml[mrow][0] = m_run;
            sm.ml[mrow][1] = l_tot;
        }
        f32x4* orow = mbuf + mrow * 32;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int jg = 0; jg < 4; ++jg) {
                f32x4 x = {o[dt][4 * jg], o[dt][4 * jg + 1], o[dt][4 * jg + 2], o[dt][4 * jg + 3]};
                orow[(dt * 8 + 2 * jg + hf) ^ ln] = x;
            }
    }
    __syncthreads();
    // 64*RB rows of 128 values leave as bf16: 16 lanes cover one 256-byte row, so a store instruction of the
    // wave writes 1 KB of consecutive memory (4 rows of a partial result; rows of the output are 256-byte runs)
#pragma unroll
    for (int k = 0; k < (kQRows * RB * 16) / kThreads; ++k) {
        const int idx = k * kThreads + tid;
        const int row_l = idx >> 4, c16 = idx & 15;       // row of the workgroup, 16-byte column of the row
        const int rs = row_l / WROWS, lr = row_l % WROWS; // row slice (wave within a stream), row inside the slice
        float mw[NS], mx = -INFINITY;
#pragma unroll
        for (int s2 = 0; s2 < NS; ++s2) { mw[s2] = sm.ml[(s2 * WPS + rs) * WROWS + lr][0]; mx = fmaxf(mx, mw[s2]); }
        const float mxs = (mx == -INFINITY) ? 0.f : mx;
        float wgt[NS], L = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < NS; ++s2) {
            wgt[s2] = __builtin_amdgcn_exp2f(mw[s2] - mxs);
            L += wgt[s2] * sm.ml[(s2 * WPS + rs) * WROWS + lr][1];
        }
        const int r = rbg * RB * kQRows + row_l;          // packed row
        const int rbo = r / kQRows, qi = r % kQRows;      // its 64-row block and row inside the block
        const bool row_live = r < n_rows;
        const int hl = row_live ? (int)(((float)r + 0.5f) * a.inv_M) : 0;
        const int i = row_live ? r - hl * M : 0, h = g * G + hl;
        // final output, or this key range's partial result: O / L in bf16 next to (max, L) in fp32
        const float inv = (L > 0.f) ? 1.f / L : 0.f;
        const int64_t blk = (((int64_t)b * a.n_chunks + chunk) * a.Hkv + g) * a.row_blocks + rbo;
        unsigned short* dst16 = (a.n_chunks == 1)
            ? out16 + (((int64_t)b * M + i) * a.Hq + h) * kD + c16 * 8
            : static_cast<unsigned short*>(a.part_o) + (blk * kQRows + qi) * kD + c16 * 8;
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s2 = 0; s2 < NS; ++s2) {
            const f32x4* prow = mbuf + ((s2 * WPS + rs) * WROWS + lr) * 32;
            acc0 += prow[(2 * c16) ^ (lr & 31)] * wgt[s2];
            acc1 += prow[(2 * c16 + 1) ^ (lr & 31)] * wgt[s2];
        }
        bf16x8 ob;
        ob[0] = (__bf16)(acc0[0] * inv); ob[1] = (__bf16)(acc0[1] * inv);
        ob[2] = (__bf16)(acc0[2] * inv); ob[3] = (__bf16)(acc0[3] * inv);
        ob[4] = (__bf16)(acc1[0] * inv); ob[5] = (__bf16)(acc1[1] * inv);
        ob[6] = (__bf16)(acc1[2] * inv); ob[7] = (__bf16)(acc1[3] * inv);
        if (row_live || a.n_chunks > 1) *reinterpret_cast<bf16x8*>(dst16) = ob;
        if (c16 == 0) {
            if (a.n_chunks == 1) {
                if (a.lse && row_live) a.lse[((int64_t)b * a.Hq + h) * M + i] = (mx + log2f(L)) * kLn2;
            } else {
                a.part_ml[(blk * kQRows + qi) * 2 + 0] = mx;
                a.part_ml[(blk * kQRows + qi) * 2 + 1] = L;
            }
        }
    }
}

// Merges the n_chunks partial results of every output row.  Grid (Hkv * ceil(G*M / 16), B): workgroup
// blockIdx.x = g + Hkv * k takes the packed rows 16k .. 16k+15 of KV head g, 16 threads per row (8 columns each,
// 16-byte loads).  With the KV head in the low part of the index a workgroup lands on the XCD whose workgroups
// wrote the partial results it reads (both kernels deal workgroups round-robin to the XCDs, KV head first).
constexpr int kCombineRows = 16;
// What the addresses of the partial results hang on comes as leading scalar arguments (preloaded into registers
// at wave start, like the main kernel's), so the loads go out without waiting for the argument block.
__global__ __launch_bounds__(256) void attn_bf16_combine_kernel(const void* part_o, const float* part_ml,
                                                                const int32_t* status, int n_chunks, int Hkv,
                                                                int row_blocks, int G, int M, float inv_M,
                                                                AttnArgs a) {
    const int g = blockIdx.x % Hkv, b = blockIdx.y;
    const int r = (blockIdx.x / Hkv) * kCombineRows + threadIdx.x / 16;      // packed row of KV head g
    if (r >= G * M) return;
    const int bad = status[b];          // requested first, looked at last: the partial loads do not wait for it
    const int hl = (int)(((float)r + 0.5f) * inv_M);              // r / M (exact for these sizes)
    const int i = r - hl * M, h = g * G + hl;
    const int d0 = (threadIdx.x % 16) * 8;
    unsigned short* dst = static_cast<unsigned short*>(a.out) + (((int64_t)b * M + i) * a.Hq + h) * kD + d0;
    const int rb = r / kQRows, qi = r % kQRows;
    const int64_t blk0 = ((int64_t)b * n_chunks * Hkv + g) * row_blocks + rb;
    const int64_t blk_step = (int64_t)Hkv * row_blocks;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float L = 0.f, mx = -INFINITY;
    for (int ch0 = 0; ch0 < n_chunks; ch0 += 8) {
        // up to 8 partials at a time: all loads of a batch are issued before any is used
        float2 ml[8];
        bf16x8 oo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t blk = blk0 + (int64_t)(ch0 + e < n_chunks ? ch0 + e : ch0) * blk_step;
            ml[e] = *reinterpret_cast<const float2*>(part_ml + (blk * kQRows + qi) * 2);
            oo[e] = *reinterpret_cast<const bf16x8*>(static_cast<const unsigned short*>(part_o) + (blk * kQRows + qi) * kD + d0);
        }
        float bm = mx;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (ch0 + e >= n_chunks) ml[e].x = -INFINITY;         // absent partials weigh nothing
            bm = fmaxf(bm, ml[e].x);
        }
        const float bms = (bm == -INFINITY) ? 0.f : bm;
        const float resc = __builtin_amdgcn_exp2f(mx - bms);        // 0 on the first batch
#pragma unroll
        for (int x = 0; x < 8; ++x) acc[x] *= resc;
        L *= resc;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float wl = __builtin_amdgcn_exp2f(ml[e].x - bms) * ml[e].y;   // the partial holds O / L
            L += wl;
#pragma unroll
            for (int x = 0; x < 8; ++x) acc[x] += wl * (float)oo[e][x];
        }
        mx = bm;
    }
    // a flagged sequence gets zeros (its workgroups wrote no partial results; what was read above is discarded)
    const float inv = bad ? 0.f : 1.f / L;
    bf16x8 ob;
#pragma unroll
    for (int x = 0; x < 8; ++x) ob[x] = (__bf16)(bad ? 0.f : acc[x] * inv);
    *reinterpret_cast<bf16x8*>(dst) = ob;
    if (a.lse && d0 == 0) a.lse[((int64_t)b * a.Hq + h) * M + i] = bad ? 0.f : (mx + log2f(L)) * kLn2;
}

template <int RB>
hipError_t launch_variant(const AttnArgs& a, hipStream_t s) {
    static std::atomic<unsigned> attr_done{0};       // one bit per device
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned bit = 1u << (dev & 31);
    if (!(attr_done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel<RB>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes<RB>());
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_release);
    }
    const dim3 grid(a.Hkv * (a.row_blocks / RB) * a.n_chunks, a.B);
    attn_bf16_kernel<RB><<<grid, 512, smem_bytes<RB>(), s>>>(a.prefix_len, a.kv_offset, a.B, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention_bf16(const AttnArgs& a, hipStream_t s) {
    hipError_t e;
    switch (a.rb_per_wg) {
        case 1: e = launch_variant<1>(a, s); break;
        case 2: e = launch_variant<2>(a, s); break;
        default: e = launch_variant<4>(a, s); break;
    }
    if (e != hipSuccess) return e;
    if (a.n_chunks > 1) {
        attn_bf16_combine_kernel<<<dim3((unsigned)(a.Hkv * ((a.G * a.M + kCombineRows - 1) / kCombineRows)), (unsigned)a.B),
                                   256, 0, s>>>(a.part_o, a.part_ml, a.status, a.n_chunks, a.Hkv, a.row_blocks, a.G, a.M,
                                                a.inv_M, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace tv
