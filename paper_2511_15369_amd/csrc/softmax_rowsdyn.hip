// Host side of the run-time-row-length slab kernel (softmax_rowsdyn.h): lane layout for a
// row length and the launch.
#include <hip/hip_runtime.h>

#include "softmax_rowsdyn.h"

namespace iptq {

// Lane layout for a row length: the fewest lanes per row that keep the blocks per lane at or
// below 8 (5 wavefronts per SIMD; measured equal or better than more blocks on fewer lanes),
// else 16 lanes per row with up to 10 blocks per lane (rows of up to about 635 scores).
// *slots is exactly ceil(most blocks a row can touch / lanes): the kernels rely on it.
// Returns false for longer rows: one wavefront per row serves those better (softmax_wide.h;
// measured 70-75 % against 66-69 % of the HBM roofline at 650 to 829 columns, 57-67 % against
// 69-75 % at 509 to 600).
bool rowsdyn_geometry(int32_t cols, int *lanes, int *slots)
{
    const int nb_max = (cols % 4 == 0) ? cols / 4 : ((cols % 2 == 0) ? (cols + 2 + 3) / 4 : (cols + 3 + 3) / 4);
    int k = 1;
    while (k < 16 && (nb_max + k - 1) / k > 8) k *= 2;
    const int n = (nb_max + k - 1) / k;
    if (n > 10) return false;
    *lanes = k;
    *slots = n;
    return true;
}

// Every row of one call if the call qualifies; returns the number of rows served through
// *done (0: not served, nothing enqueued).
hipError_t softmax_rowsdyn_launch(const SoftmaxCall &c, int32_t cols, int post_mode, int64_t *done,
                                  hipStream_t stream)
{
    *done = 0;
    int k = 0, slots = 0;
    if (!rowsdyn_geometry(cols, &k, &slots)) return hipSuccess;
    const int rpw = 64 / k;
    const bool has_bias = c.bias != nullptr;
    const bool aligned = ((reinterpret_cast<uintptr_t>(c.scores) | reinterpret_cast<uintptr_t>(c.bias)) & 3) == 0;
    const bool bias_ok = !has_bias || ((int64_t)c.P.bias_period_rows * cols >= 4 &&
                                       (int64_t)c.P.bias_period_rows * cols < ((int64_t)1 << 31) &&
                                       c.P.bias_period_rows >= rpw);
    const int64_t n_slabs = (c.rows + rpw - 1) / rpw;
    if (!aligned || !bias_ok || n_slabs == 0) return hipSuccess;
    DynArgs A;
    A.scores = c.scores; A.bias = c.bias; A.out = c.out;
    A.n_slabs = n_slabs; A.tail_rows = (int32_t)(c.rows % rpw);
    A.cols = cols; A.post_mode = post_mode;
    A.wave_lds = (int32_t)((((int64_t)rpw * cols * 4 + 15) & ~(int64_t)15) + kPostLutBytes);
    A.P = c.P;
    int wpb = 65536 / A.wave_lds;                     // wavefronts per workgroup: 1..4
    if (wpb > 4) wpb = 4;
    if (wpb < 1) return hipSuccess;
    int64_t n_wgs = (n_slabs + wpb - 1) / wpb;
    A.share_q = 0; A.share_magic = 0; A.share_sh = 0;
    if (has_bias && wpb > 1) {
        int64_t a = c.P.bias_period_rows, b = rpw;
        while (b != 0) { const int64_t t = a % b; a = b; b = t; }              // a = gcd
        const int64_t q = c.P.bias_period_rows / a;
        if (q >= 2 && q < 65536 && q * wpb <= n_slabs &&
            make_magic_u32((uint32_t)q, 31, &A.share_magic, &A.share_sh)) {
            A.share_q = (uint32_t)q;
            n_wgs = (n_slabs + (int64_t)wpb * q - 1) / ((int64_t)wpb * q) * q;
        }
    }
    const dim3 grid((unsigned)n_wgs), block(64 * wpb);
    const size_t lds = (size_t)A.wave_lds * wpb;
    bool launched;
    if (k == 1) launched = rowsdyn_launch_k1(A, slots, c.P.mode16, grid, block, lds, stream);
    else if (k == 2) launched = rowsdyn_launch_k2(A, slots, c.P.mode16, grid, block, lds, stream);
    else if (k == 4) launched = rowsdyn_launch_k4(A, slots, c.P.mode16, grid, block, lds, stream);
    else if (k == 8) launched = rowsdyn_launch_k8(A, slots, c.P.mode16, grid, block, lds, stream);
    else launched = slots <= 8 ? rowsdyn_launch_k16(A, slots, c.P.mode16, grid, block, lds, stream)
                               : rowsdyn_launch_k16_long(A, slots, c.P.mode16, grid, block, lds, stream);
    if (!launched) return hipSuccess;                 // no such layout: the caller's next kernel serves it
    *done = c.rows;
    return hipGetLastError();
}

}  // namespace iptq
