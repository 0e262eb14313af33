// Tree preparation: the ancestor mask of a verification step, built once and shared by every layer's
// attention call (Section 3.1 / Figure 4: the mask belongs to the step, not to a layer).
#include "tv_internal.hpp"

namespace tv {

namespace {

// One workgroup per sequence, one thread per row: the same checks and the same ancestor walk the attention
// kernels run when no prepared tree is handed over.
__global__ __launch_bounds__(kMaxRows) void prepare_tree_kernel(const int32_t* parent, const uint8_t* kind, int M,
                                                                PreparedTree* out) {
    __shared__ int s_parent[kMaxRows];
    __shared__ unsigned char s_kind[kMaxRows];
    __shared__ int s_flag;
    const int b = blockIdx.x, i = threadIdx.x;
    if (i < M) {
        s_parent[i] = parent[(int64_t)b * M + i];
        s_kind[i] = kind[(int64_t)b * M + i];
    }
    __syncthreads();
    const int bad = validate_tree(s_parent, s_kind, M, &s_flag);
    PreparedTree& t = out[b];
    unsigned long long w0 = 0, w1 = 0;
    if (i < M && !bad) ancestor_bits(s_parent, i, &w0, &w1);
    t.bits[i][0] = w0;                       // rows past M: zeros
    t.bits[i][1] = w1;
    t.kind[i] = (i < M) ? s_kind[i] : (unsigned char)TV_KIND_NODE;
    if (i == 0) t.status = bad;
}

}  // namespace

hipError_t launch_prepare_tree(const int32_t* parent, const uint8_t* kind, int B, int M, PreparedTree* out, hipStream_t s) {
    prepare_tree_kernel<<<dim3((unsigned)B), kMaxRows, 0, s>>>(parent, kind, M, out);
    return hipGetLastError();
}

}  // namespace tv
