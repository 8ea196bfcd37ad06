// Multi-query-row causal decode attention against the contiguous KV cache ("attention" in Section 3's
// cost breakdown; the cache is the one of Sections 2 and 4.2).
//
// For sequence b, head h, the M = K+1 new rows (row i at absolute position L_b + i) attend cache
// positions 0..L_b + i; the rows' own keys/values were appended before this kernel runs, so everything
// is read back from the cache.  The KV range is split over workgroups (grid.x) and, inside a
// workgroup, over 4 wavefronts; every key/value tile is read from HBM exactly once and serves all M
// rows: the M query rows are the 16-wide B operand of the MFMAs (held in registers), keys and
// (block-transposed) values are the streamed A operand, 16 bytes per lane.
//
//   S^T[pos][m]  = sum_e K[pos][e] * Q[m][e]        (keys as A, queries as B)
//   O^T[e][m]   += sum_pos V^T[e][pos] * P[m][pos]  (transposed values as A, softmax weights as B)
//
// The row order of a key tile is permuted so that the score registers a lane receives are exactly
// the 8 (bf16) or 4 (f32) consecutive positions it must supply as the B operand of the P.V product:
// tile t, row i  <->  position p0 + (i/4)*E + 4t + (i%4).
// Online softmax in the log2 domain per wave; waves, then splits, are merged by log-sum-exp in a
// fixed order.  The second kernel merges the splits, normalises and writes the result as the
// activation planes the O projection consumes.
#include "attention_core.h"

namespace ss {

// merge over splits, normalise, write activation planes: grid (R, H), block HD
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    __shared__ AttnSmem<HD, 4> sm;
    attn_unit<T, HD, 4>(a, blockIdx.x, blockIdx.y, blockIdx.z, a.len[blockIdx.z], sm);
}

// a single split: the workgroup normalises and writes the activation planes itself (no partials, no merge launch)
template <typename T, int HD, int NWX = 4>
__global__ __launch_bounds__(NWX * 64) void attn_direct_kernel(AttnArgs a) {
    __shared__ AttnSmem<HD, NWX> sm;
    attn_unit<T, HD, NWX, false, true>(a, 0, blockIdx.y, blockIdx.z, a.len[blockIdx.z], sm);
}

template <typename T>
__global__ void attn_merge_kernel(AttnArgs a) {
    const int row = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
    ActPlanes<T> out{reinterpret_cast<T *>(a.act_out), a.act_out_plane, a.ld_out};
    store_act(out, (size_t)row * a.ld_out + h * a.hd + e, attn_merge_elem<false>(a, row, h, e));
}

template <typename T> static void launch_attention_t(const AttnArgs &a, hipStream_t st) {
    dim3 grid(a.nsplit, a.H, a.B);
    if (a.nsplit == 1) {
        // few units with a short context (one split by the host's choice): 8 waves, so that a wave has one step up to 256 positions
        if (a.hd == 128 && a.B * a.H < 256) {
            hipLaunchKernelGGL((attn_direct_kernel<T, 128, 8>), grid, dim3(512), 0, st, a);
            return;
        }
        if (a.hd == 128) hipLaunchKernelGGL((attn_direct_kernel<T, 128>), grid, dim3(256), 0, st, a);
        else if (a.hd == 64) hipLaunchKernelGGL((attn_direct_kernel<T, 64>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_direct_kernel<T, 32>), grid, dim3(256), 0, st, a);
        return;
    }
    if (a.hd == 128) hipLaunchKernelGGL((attn_partial_kernel<T, 128>), grid, dim3(256), 0, st, a);
    else if (a.hd == 64) hipLaunchKernelGGL((attn_partial_kernel<T, 64>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_partial_kernel<T, 32>), grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((attn_merge_kernel<T>), dim3(a.R, a.H), dim3(a.hd), 0, st, a);
}

void launch_attention(int dtype, const AttnArgs &a, hipStream_t st) {
    if (dtype) launch_attention_t<bf16_t>(a, st);
    else launch_attention_t<float>(a, st);
}

} // namespace ss
