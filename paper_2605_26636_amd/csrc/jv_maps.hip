// Window / padding index maps (Sec. 3.2.2 of the paper: non-overlapping windows
// on the token grid), on the host and as a kernel.  Integer arithmetic only.
#include "jv_common.h"

namespace jv {

// One padded-grid cell -> (window, slot, token or -1).  Shared by the host loop
// and the kernel so both write identical bytes.
__host__ __device__ inline void map_cell(int r, int c, int H, int W, int wh, int ww, int wins_x,
                                         int *win, int *slot, int *token) {
    *win = (r / wh) * wins_x + (c / ww);
    *slot = (r % wh) * ww + (c % ww);
    *token = (r < H && c < W) ? r * W + c : -1;
}

__global__ void window_maps_kernel(WindowGeom g, int32_t *token_index, uint8_t *pad_mask,
                                   int32_t *window_of_token) {
    const int cells = g.Hp * g.Wp;
    for (int cell = blockIdx.x * blockDim.x + threadIdx.x; cell < cells;
         cell += gridDim.x * blockDim.x) {
        int r = cell / g.Wp, c = cell % g.Wp, win, slot, token;
        map_cell(r, c, g.H, g.W, g.wh, g.ww, g.wins_x, &win, &slot, &token);
        size_t at = (size_t)win * g.slots + slot;
        if (token_index) token_index[at] = token;
        if (pad_mask) pad_mask[at] = token >= 0 ? 1 : 0;
        if (window_of_token && token >= 0) window_of_token[token] = win;
    }
}

}  // namespace jv

extern "C" {

jv_status jv_window_maps_host(int32_t grid_h, int32_t grid_w, int32_t win_h, int32_t win_w,
                              int32_t *token_index, uint8_t *pad_mask, int32_t *window_of_token) {
    jv::clear_error();
    jv::WindowGeom g;
    jv_status st = jv::make_window_geom(grid_h, grid_w, win_h, win_w, &g);
    if (st != JV_OK) return st;
    for (int r = 0; r < g.Hp; ++r)
        for (int c = 0; c < g.Wp; ++c) {
            int win, slot, token;
            jv::map_cell(r, c, g.H, g.W, g.wh, g.ww, g.wins_x, &win, &slot, &token);
            size_t at = (size_t)win * g.slots + slot;
            if (token_index) token_index[at] = token;
            if (pad_mask) pad_mask[at] = token >= 0 ? 1 : 0;
            if (window_of_token && token >= 0) window_of_token[token] = win;
        }
    return JV_OK;
}

jv_status jv_window_maps_device(int32_t grid_h, int32_t grid_w, int32_t win_h, int32_t win_w,
                                int32_t *token_index, uint8_t *pad_mask,
                                int32_t *window_of_token, void *hip_stream) {
    jv::clear_error();
    jv::WindowGeom g;
    jv_status st = jv::make_window_geom(grid_h, grid_w, win_h, win_w, &g);
    if (st != JV_OK) return st;
    if (!token_index && !pad_mask && !window_of_token) return JV_OK;
    const int cells = g.Hp * g.Wp;
    int blocks = (cells + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(jv::window_maps_kernel, dim3(blocks), dim3(256), 0,
                       (hipStream_t)hip_stream, g, token_index, pad_mask, window_of_token);
    return jv::launch_status("window_maps_kernel");
}

}  // extern "C"
