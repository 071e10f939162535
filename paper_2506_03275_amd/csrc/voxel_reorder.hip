// Voxel token reorder and its inverse (Alg. 1; Sec. 3.2.1) for gfx950.
//
// The permutation has a closed form, so no index table is read: every wave
// computes the source (or destination) row of its token from the grid geometry
// and moves the row with 128-bit (or 32-bit) accesses.  The copy touches each
// byte once on the way in and once on the way out: it is bound by HBM.
#include "common.h"

namespace chipmunk {

struct VoxelGeom {
    int n_prefix, T, H, W, n_suffix;
    int vt, vh, vw;
    int Tf, Hf, Wf;   // extent covered by full voxels in each dimension
    int n_full;       // tokens inside full voxels
    int grid;         // T*H*W
    int N;
};

// position before the reorder of the token that sits at position i after it
__device__ __forceinline__ int voxel_old_position(const VoxelGeom& g, int i) {
    if (i < g.n_prefix) return i;
    int j = i - g.n_prefix;
    if (j >= g.grid) return i;  // suffix
    int t, h, w;
    if (j < g.n_full) {
        int vol = g.vt * g.vh * g.vw;
        int v = j / vol, r = j - v * vol;
        int wc_n = g.Wf / g.vw, hc_n = g.Hf / g.vh;
        int wc = v % wc_n, hc = (v / wc_n) % hc_n, tc = v / (wc_n * hc_n);
        int dw = r % g.vw, dh = (r / g.vw) % g.vh, dt = r / (g.vw * g.vh);
        t = tc * g.vt + dt;
        h = hc * g.vh + dh;
        w = wc * g.vw + dw;
    } else {
        // remainder, in raster order: inside a frame t < Tf the rows h < Hf give their
        // columns w >= Wf, then the rows h >= Hf are whole; frames t >= Tf are whole.
        int rho = j - g.n_full;
        int edge = g.Hf * (g.W - g.Wf);
        int per_frame = edge + (g.H - g.Hf) * g.W;
        int in_frames = g.Tf * per_frame;
        if (rho < in_frames) {
            t = rho / per_frame;
            int r = rho - t * per_frame;
            if (r < edge) {
                h = r / (g.W - g.Wf);
                w = g.Wf + (r - h * (g.W - g.Wf));
            } else {
                r -= edge;
                h = g.Hf + r / g.W;
                w = r % g.W;
            }
        } else {
            int r = rho - in_frames;
            t = g.Tf + r / (g.H * g.W);
            r = r % (g.H * g.W);
            h = r / g.W;
            w = r % g.W;
        }
    }
    return g.n_prefix + (t * g.H + h) * g.W + w;
}

__global__ __launch_bounds__(256) void voxel_perm_kernel(VoxelGeom g, int32_t* perm, int32_t* inv_perm) {
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= g.N) return;
    int old = voxel_old_position(g, i);
    if (perm) perm[i] = old;
    if (inv_perm) inv_perm[old] = i;
}

// One wave moves one row at a time.  VEC is uint4 (16-byte words) or uint32_t.
template <typename VEC>
__global__ __launch_bounds__(256) void voxel_copy_kernel(VoxelGeom g, const VEC* __restrict__ src,
                                                         VEC* __restrict__ dst, int64_t total_rows,
                                                         int words_per_row, int inverse) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t row = wave; row < total_rows; row += nwaves) {
        int b = (int)(row / g.N);
        int i = (int)(row - (int64_t)b * g.N);
        int old = voxel_old_position(g, i);
        int64_t from = (int64_t)b * g.N + (inverse ? i : old);
        int64_t to = (int64_t)b * g.N + (inverse ? old : i);
        const VEC* s = src + from * words_per_row;
        VEC* d = dst + to * words_per_row;
        for (int x = lane; x < words_per_row; x += 64) d[x] = s[x];
    }
}

}  // namespace chipmunk

using namespace chipmunk;

extern "C" int32_t chipmunk_voxel_reorder(const void* src, void* dst, int32_t* perm, int32_t* inv_perm,
                                          int batch, int n_prefix, int T, int H, int W, int n_suffix,
                                          int vt, int vh, int vw, int row_bytes, int inverse, void* stream) {
    if ((src == nullptr) != (dst == nullptr)) return CHIPMUNK_ERR_NULL;
    if (!src && !perm && !inv_perm) return CHIPMUNK_ERR_NULL;
    if (n_prefix < 0 || n_suffix < 0 || T < 1 || H < 1 || W < 1 || vt < 1 || vh < 1 || vw < 1)
        return CHIPMUNK_ERR_SHAPE;
    int64_t N64 = (int64_t)n_prefix + (int64_t)T * H * W + n_suffix;
    if (N64 > 0x7fffffffLL) return CHIPMUNK_ERR_SHAPE;
    if (src && (batch < 1 || row_bytes < 1)) return CHIPMUNK_ERR_SHAPE;
    if (src && (row_bytes % 4) != 0) return CHIPMUNK_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(perm) & 3u) || (reinterpret_cast<uintptr_t>(inv_perm) & 3u) ||
        (reinterpret_cast<uintptr_t>(src) & 3u) || (reinterpret_cast<uintptr_t>(dst) & 3u))
        return CHIPMUNK_ERR_ALIGN;
    if (src) {  // the two buffers must not overlap
        const char* s0 = (const char*)src;
        const char* d0 = (const char*)dst;
        int64_t bytes = (int64_t)batch * N64 * row_bytes;
        if (s0 < d0 + bytes && d0 < s0 + bytes) return CHIPMUNK_ERR_SHAPE;
    }
    VoxelGeom g;
    g.n_prefix = n_prefix; g.T = T; g.H = H; g.W = W; g.n_suffix = n_suffix;
    g.vt = vt; g.vh = vh; g.vw = vw;
    g.Tf = (T / vt) * vt; g.Hf = (H / vh) * vh; g.Wf = (W / vw) * vw;
    g.n_full = g.Tf * g.Hf * g.Wf;
    g.grid = T * H * W;
    g.N = (int)N64;
    hipStream_t s = (hipStream_t)stream;
    if (perm || inv_perm) {
        hipLaunchKernelGGL(voxel_perm_kernel, dim3((g.N + 255) / 256), dim3(256), 0, s, g, perm, inv_perm);
        if (launch_status() != CHIPMUNK_OK) return CHIPMUNK_ERR_LAUNCH;
    }
    if (src) {
        int64_t total_rows = (int64_t)batch * g.N;
        int64_t blocks = (total_rows + 3) / 4;
        if (blocks > 256 * 64) blocks = 256 * 64;  // 64 resident-sized groups per CU, rows strided over them
        if (row_bytes % 16 == 0 && aligned16(src) && aligned16(dst))
            hipLaunchKernelGGL((voxel_copy_kernel<uint4>), dim3((unsigned)blocks), dim3(256), 0, s, g,
                               (const uint4*)src, (uint4*)dst, total_rows, row_bytes / 16, inverse);
        else
            hipLaunchKernelGGL((voxel_copy_kernel<uint32_t>), dim3((unsigned)blocks), dim3(256), 0, s, g,
                               (const uint32_t*)src, (uint32_t*)dst, total_rows, row_bytes / 4, inverse);
        if (launch_status() != CHIPMUNK_OK) return CHIPMUNK_ERR_LAUNCH;
    }
    return CHIPMUNK_OK;
}
