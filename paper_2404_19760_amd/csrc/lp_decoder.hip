// The paper's two-MLP decoder (opacity MLP and view-dependent feature MLP, Section 3.3) is run
// as ONE block-structured MLP, so that the Renderer kernels stay single-MLP kernels: these
// two small kernels build the merged weights from the caller's two MLPs before a launch and
// hand the merged gradient back to the two MLPs' gradient buffers after a backward.
#include "lp_kernels.h"

namespace lp {

namespace {

struct Source {
    int which;   // 0: constant `value`; 1: opacity MLP; 2: feature MLP
    int layer;   // source layer
    int index;   // element of W[layer] (or of b[layer] when `bias`)
    bool bias;
    float value;
};

__host__ __device__ inline int hidden_width(const int* dims, int LX, int l) { return dims[l + 1 < LX - 1 ? l + 1 : LX - 1]; }
__host__ __device__ inline int out_width(const int* dims, int LX, int L, int l)
{
    return l == L - 1 ? dims[LX] : hidden_width(dims, LX, l);
}

// Where element (row o, column k) of combined layer l comes from; k < 0: the bias of row o.
__device__ Source dec_source(const DecLayout& d, int l, int o, int k)
{
    Source src = {0, 0, 0, k < 0, 0.0f};
    const int rows_s = out_width(d.dims_s, d.Ls, d.L, l);
    const bool is_s = o < rows_s;
    const int* dims = is_s ? d.dims_s : d.dims_v;
    const int LX = is_s ? d.Ls : d.Lv;
    const int r = is_s ? o : o - rows_s;
    // this MLP's input columns of the combined layer
    int col0, ncol;
    if (l == 0) { col0 = 0; ncol = is_s ? d.C : d.C + d.E; }
    else {
        const int in_s = out_width(d.dims_s, d.Ls, d.L, l - 1);
        col0 = is_s ? 0 : in_s;
        ncol = is_s ? in_s : out_width(d.dims_v, d.Lv, d.L, l - 1);
    }
    if (k >= 0 && (k < col0 || k >= col0 + ncol)) return src;   // structural zero
    const int kk = k - col0;
    int sl;
    if (l == d.L - 1) sl = LX - 1;        // the MLP's output layer
    else if (l < LX - 1) sl = l;          // one of its hidden layers
    else {                                // carried: identity block, zero bias
        src.value = (k >= 0 && kk == r) ? 1.0f : 0.0f;
        return src;
    }
    src.which = is_s ? 1 : 2;
    src.layer = sl;
    src.index = k < 0 ? r : r * dims[sl] + kk;
    return src;
}

// (layer, row, column or -1) of combined parameter i
__device__ bool param_position(const MlpDev& m, int i, int& l, int& o, int& k)
{
    for (l = 0; l < m.n_layers; ++l) {
        const int nin = m.dims[l], nw = nin * m.dims[l + 1];
        if (i >= m.w_off[l] && i < m.w_off[l] + nw) {
            o = (i - m.w_off[l]) / nin;
            k = (i - m.w_off[l]) - o * nin;
            return true;
        }
        if (i >= m.b_off[l] && i < m.b_off[l] + m.dims[l + 1]) {
            o = i - m.b_off[l];
            k = -1;
            return true;
        }
    }
    return false;
}

__global__ void dec_pack_kernel(DecLayout d, MlpDev m, float* packed, float* grads)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= m.param_total) return;
    int l, o, k;
    float v = 0.0f;
    if (param_position(m, i, l, o, k)) {
        const Source s = dec_source(d, l, o, k);
        if (s.which == 0) v = s.value;
        else if (s.which == 1) v = s.bias ? d.bs[s.layer][s.index] : d.Ws[s.layer][s.index];
        else v = s.bias ? d.bv[s.layer][s.index] : d.Wv[s.layer][s.index];
    }
    packed[i] = v;
    if (grads) grads[i] = 0.0f;
}

__global__ void dec_unpack_kernel(DecLayout d, MlpDev m, const float* grads)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= m.param_total) return;
    int l, o, k;
    if (!param_position(m, i, l, o, k)) return;
    const Source s = dec_source(d, l, o, k);
    if (s.which == 0) return;   // zero and identity blocks have no parameter behind them
    float* dst = s.which == 1 ? (s.bias ? d.dbs[s.layer] : d.dWs[s.layer]) : (s.bias ? d.dbv[s.layer] : d.dWv[s.layer]);
    dst[s.index] += grads[i];   // every source parameter appears exactly once in the merged MLP
}

}  // namespace

void dec_combined_dims(const DecLayout& d, int in_width, int dims[LP_MAX_LAYERS + 1])
{
    dims[0] = in_width;
    for (int l = 0; l < d.L; ++l) dims[l + 1] = out_width(d.dims_s, d.Ls, d.L, l) + out_width(d.dims_v, d.Lv, d.L, l);
}

hipError_t launch_dec_pack(const DecLayout& d, const MlpDev& m, float* packed, float* grads, hipStream_t stream)
{
    const int threads = 256;
    hipLaunchKernelGGL(dec_pack_kernel, dim3((m.param_total + threads - 1) / threads), dim3(threads), 0, stream, d, m,
                       packed, grads);
    return hipGetLastError();
}

hipError_t launch_dec_unpack(const DecLayout& d, const MlpDev& m, const float* grads, hipStream_t stream)
{
    const int threads = 256;
    hipLaunchKernelGGL(dec_unpack_kernel, dim3((m.param_total + threads - 1) / threads), dim3(threads), 0, stream, d,
                       m, grads);
    return hipGetLastError();
}

}  // namespace lp
