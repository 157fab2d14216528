// Packing of the kept visual K/V rows into a contiguous region (paper section 3.2: the selected
// visual KV entries are packed contiguously so that the decode attention of the following tokens
// reads no irregular pattern).  k_pack/v_pack[b, g, i, :] = k_vis/v_vis[b, g, idx[b,g,i], :] for
// i < count[b,g]; the rows from count[b,g] to k are zero-filled.  A pure byte copy: a row is moved as
// 16-byte pieces, one per lane, so a wavefront load or store covers whole rows.
#include "sv_kernels.h"

namespace sv {
namespace {

constexpr int kPackThreads = 256;

__global__ __launch_bounds__(kPackThreads) void pack_kernel(const PackArgs a) {
    const int g = blockIdx.y, b = blockIdx.z;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int lpr = a.row_bytes / 16;                      // lanes per row
    const int rows_per_pass = kPackThreads / lpr;
    const int c = threadIdx.x % lpr, r_in = threadIdx.x / lpr;
    int cnt = a.count[unit];
    cnt = cnt < 0 ? 0 : (cnt < a.k ? cnt : a.k);
    const int32_t* idx_row = a.idx + unit * a.k;
    const char* ks = static_cast<const char*>(a.k_vis) + ((int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh) * a.elem;
    const char* vs = static_cast<const char*>(a.v_vis) + ((int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh) * a.elem;
    char* kd = static_cast<char*>(a.k_pack) + unit * a.k * (int64_t)a.row_bytes;
    char* vd = static_cast<char*>(a.v_pack) + unit * a.k * (int64_t)a.row_bytes;
    const int i0 = blockIdx.x * a.rows_per_block;
    const int i1 = min(i0 + a.rows_per_block, a.k);
    for (int i = i0 + r_in; i < i1; i += rows_per_pass) {
        uint4 kv = make_uint4(0u, 0u, 0u, 0u), vv = kv;
        if (i < cnt) {
            int j = idx_row[i];
            j = j < 0 ? 0 : (j < a.n_vis_max ? j : a.n_vis_max - 1);   // a faulty idx must not fault the GPU
            const int64_t off = (int64_t)j * a.vis_sn * a.elem + c * 16;
            kv = *reinterpret_cast<const uint4*>(ks + off);
            vv = *reinterpret_cast<const uint4*>(vs + off);
        }
        *reinterpret_cast<uint4*>(kd + (int64_t)i * a.row_bytes + c * 16) = kv;
        *reinterpret_cast<uint4*>(vd + (int64_t)i * a.row_bytes + c * 16) = vv;
    }
}

}  // namespace

hipError_t launch_pack(const PackArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0 || a.k == 0) return hipSuccess;
    PackArgs p = a;
    p.rows_per_block = 128;
    dim3 grid((unsigned)((a.k + p.rows_per_block - 1) / p.rows_per_block), (unsigned)a.Hkv, (unsigned)a.B);
    hipLaunchKernelGGL(pack_kernel, grid, dim3(kPackThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace sv
