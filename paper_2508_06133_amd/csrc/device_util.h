// Device helpers shared by the timeline kernels: wavefront reductions and the mapping from a
// position of a candidate order to a request id.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kvsched.h"

namespace {

constexpr int WAVE = 64;

template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}

// Maximum over the 64 lanes; all lanes must be active.  Four DPP steps leave every lane of a
// 16-lane row with the row's maximum (quad swaps, then mirror within 8 and within 16); the
// four row results are combined on the scalar unit.
__device__ __forceinline__ int wave_max_i32(int v)
{
    v = max(v, dpp_mov<0xB1>(v));   // quad_perm [1,0,3,2]
    v = max(v, dpp_mov<0x4E>(v));   // quad_perm [2,3,0,1]
    v = max(v, dpp_mov<0x141>(v));  // row_half_mirror
    v = max(v, dpp_mov<0x140>(v));  // row_mirror
    const int a = __builtin_amdgcn_readlane(v, 0);
    const int b = __builtin_amdgcn_readlane(v, 16);
    const int c = __builtin_amdgcn_readlane(v, 32);
    const int d = __builtin_amdgcn_readlane(v, 48);
    return max(max(a, b), max(c, d));
}

// Position k of candidate order -> request id.
template <bool MOVES>
struct OrderReader {
    const int32_t *row;  // explicit row, or the base order
    int mt, mi, mj;      // the move (MOVES only)

    __device__ __forceinline__ int at(int k) const
    {
        if (!MOVES) return row[k];
        int pos = k;
        if (mt == KVSCHED_MOVE_SWAP) {
            pos = (k == mi) ? mj : ((k == mj) ? mi : k);
        } else if (mi < mj) {  // entry i moves back to j; (i, j] shift forward by one
            if (k >= mi && k <= mj) pos = (k == mj) ? mi : k + 1;
        } else {  // entry i moves up to j; [j, i) shift back by one
            if (k >= mj && k <= mi) pos = (k == mj) ? mi : k - 1;
        }
        return row[pos];
    }
};

}  // namespace
