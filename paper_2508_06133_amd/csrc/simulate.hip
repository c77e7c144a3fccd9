// Timeline kernels: Phase 2 of Algorithm 1 ("Scheduling Execution") for many candidate
// orders at once, one 64-lane wavefront per candidate, plus the small kernels around it
// (length scan, order / move validation, argmin over candidates).
//
// Per-timeline state is the future-memory profile P(tau) = memory held at round tau by the
// requests admitted so far (the quantity M(X, t*) of Section 4), kept for the next H rounds
// in a ring of H int32 slots in LDS (H = power of two >= the longest decode length).
//
// Because admission is strictly in order and stops at the first request that does not fit
// (Algorithm 1's `break`), the start round of the k-th request of an order is the smallest
// t >= (start of the (k-1)-th) at which it fits beside everything admitted before it.  For a
// request (s, o), round tau rules out exactly the starts t with tau - o <= t <= tau - 1 and
// t < P(tau) + s + tau - M (Eq. 1 rearranged), so the search scans the window (t, t + o],
// moves t to the largest bound any scanned round imposes, and only has to look at the
// rounds that entered the window since.  Each round is therefore inspected once per request
// (o + waited rounds), then the admitted request's own ramp s+1..s+o is added to the ring.
#include "kvsched_internal.h"
#include "device_util.h"

#include <limits.h>

namespace {

template <int H, int WPB, bool MOVES>
__global__ __launch_bounds__(WAVE *WPB) void timeline_kernel(SimParams p)
{
    __shared__ int ring_all[H * WPB];
    const int lane = threadIdx.x & (WAVE - 1);
    const int cand = __builtin_amdgcn_readfirstlane(blockIdx.x * WPB + (threadIdx.x >> 6));
    if (cand >= p.C) return;
    int *ring = ring_all + (threadIdx.x >> 6) * H;
    for (int i = lane; i < H; i += WAVE) ring[i] = 0;

    const int n = p.n;
    const int M = p.M;
    OrderReader<MOVES> rd;
    if (MOVES) {
        rd.row = p.src.base;
        rd.mt = KVSCHED_MOVE_SWAP;
        rd.mi = rd.mj = 0;
        if (cand < p.C - 1) {  // the last timeline is the base order itself
            rd.mt = p.src.moves[3 * (size_t)cand];
            rd.mi = min(max(p.src.moves[3 * (size_t)cand + 1], 0), n - 1);
            rd.mj = min(max(p.src.moves[3 * (size_t)cand + 2], 0), n - 1);
        }
    } else {
        rd.row = p.src.orders + (size_t)cand * (size_t)n;
        rd.mt = rd.mi = rd.mj = 0;
    }
    int32_t *crow = p.completion_out ? p.completion_out + (size_t)cand * (size_t)n : nullptr;

    long long tel = 0;
    int t = 0;  // start round of the previous request in the order
    __builtin_amdgcn_wave_barrier();

    for (int k0 = 0; k0 < n; k0 += WAVE) {
        // 64 positions of the order at a time: ids read coalesced, lengths gathered
        const int k = k0 + lane;
        int r = 0, sv = 1, ov = 1;
        if (k < n) {
            r = min(max(rd.at(k), 0), n - 1);
            sv = p.s[r];
            ov = p.o[r];
        }
        const bool bad = (sv < 1) | (ov < 1) | (ov > p.o_bound) | ((long long)sv + (long long)ov > (long long)M);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // cannot be scheduled: report, do not loop forever
            if (lane == 0) p.tel_out[cand] = -1;
            return;
        }
        const int cnt = min(WAVE, n - k0);
        int cv = 0;  // completion round of position k0 + lane
        for (int j = 0; j < cnt; ++j) {
            const int sj = __builtin_amdgcn_readlane(sv, j);
            const int oj = __builtin_amdgcn_readlane(ov, j);
            const int bias = sj - M;
            int lo = t + 1;
            for (;;) {
                const int hi = t + oj;
                int acc = INT_MIN;
                for (int tau0 = lo; tau0 <= hi; tau0 += WAVE) {
                    const int tau = tau0 + lane;
                    if (tau <= hi) {
                        const int need = ring[tau & (H - 1)] + bias + tau;  // least start round tau allows
                        acc = max(acc, min(tau, need));                      // tau constrains only t < tau
                    }
                }
                const int tn = wave_max_i32(acc);
                if (tn <= t) break;
                // rounds (t, tn] are behind every later start: their slots become rounds + H
                for (int tau0 = t + 1; tau0 <= tn; tau0 += WAVE) {
                    const int tau = tau0 + lane;
                    if (tau <= tn) ring[tau & (H - 1)] = 0;
                }
                __builtin_amdgcn_wave_barrier();
                lo = hi + 1;
                t = tn;
            }
            // admitted at round t: holds sj + a tokens at round t + a
            for (int tau0 = t + 1; tau0 <= t + oj; tau0 += WAVE) {
                const int tau = tau0 + lane;
                if (tau <= t + oj) ring[tau & (H - 1)] += sj + (tau - t);
            }
            __builtin_amdgcn_wave_barrier();
            const int c = t + oj;
            tel += c;
            cv = (lane == j) ? c : cv;
        }
        if (crow && k < n) crow[p.completion_by_position ? k : r] = cv;
    }
    if (lane == 0) p.tel_out[cand] = tel;
}

// One block: largest decode length and well-formedness of (s, o); resets the status word.
__global__ __launch_bounds__(1024) void scan_lengths_kernel(const int32_t *s, const int32_t *o, int32_t n, int32_t M,
                                                            int32_t o_bound, int32_t *words)
{
    __shared__ int sh_max[16];
    __shared__ int sh_flag[16];
    int mx = 0, flag = 0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const int sv = s[i], ov = o[i];
        mx = max(mx, ov);
        if (sv < 1 || ov < 1 || (long long)sv + (long long)ov > (long long)M) flag |= KVSCHED_DEV_BAD_LENGTH;
        if (o_bound > 0 && ov > o_bound) flag |= KVSCHED_DEV_O_MAX;
    }
    mx = wave_max_i32(mx);
    flag = wave_max_i32(flag & 1) | wave_max_i32(flag & KVSCHED_DEV_O_MAX);
    if ((threadIdx.x & 63) == 0) {
        sh_max[threadIdx.x >> 6] = mx;
        sh_flag[threadIdx.x >> 6] = flag;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) {
            mx = max(mx, sh_max[w]);
            flag |= sh_flag[w];
        }
        words[KVS_W_STATUS] = flag;
        words[KVS_W_OMAX] = mx;
        words[KVS_W_MINPOS] = INT_MAX;
        words[KVS_W_MAXPOS] = -1;
    }
}

// One wavefront per row: is it a permutation of 0..n-1?  Bitmap of n bits per wave in LDS.
template <int WPB>
__global__ __launch_bounds__(WAVE *WPB) void check_orders_kernel(const int32_t *orders, int32_t C, int32_t n,
                                                                 int64_t *tel_out, int32_t *words)
{
    extern __shared__ unsigned int bitmap_all[];
    const int lane = threadIdx.x & (WAVE - 1);
    const int cand = blockIdx.x * WPB + (threadIdx.x >> 6);
    if (cand >= C) return;
    const int nw = (n + 31) >> 5;
    unsigned int *bm = bitmap_all + (size_t)(threadIdx.x >> 6) * nw;
    for (int i = lane; i < nw; i += WAVE) bm[i] = 0;
    __builtin_amdgcn_wave_barrier();
    const int32_t *row = orders + (size_t)cand * (size_t)n;
    bool bad = false;
    for (int k = lane; k < n; k += WAVE) {
        const int r = row[k];
        if (r < 0 || r >= n) {
            bad = true;
        } else {
            const unsigned int bit = 1u << (r & 31);
            if (atomicOr(&bm[r >> 5], bit) & bit) bad = true;
        }
    }
    if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) {
        tel_out[cand] = -1;
        atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_ORDER);
    }
}

// The same for long rows: one workgroup of 1024 threads per row (a single wavefront would walk a row of
// 100000 entries in 1563 dependent turns).
__global__ __launch_bounds__(1024) void check_orders_wide_kernel(const int32_t *orders, int32_t C, int32_t n,
                                                                 int64_t *tel_out, int32_t *words)
{
    extern __shared__ unsigned int bitmap_all[];
    const int cand = blockIdx.x;
    const int nw = (n + 31) >> 5;
    for (int i = threadIdx.x; i < nw; i += 1024) bitmap_all[i] = 0;
    __syncthreads();
    const int32_t *row = orders + (size_t)cand * (size_t)n;
    int bad = 0;
    for (int k = threadIdx.x; k < n; k += 1024) {
        const int r = row[k];
        if (r < 0 || r >= n) {
            bad = 1;
        } else {
            const unsigned int bit = 1u << (r & 31);
            if (atomicOr(&bitmap_all[r >> 5], bit) & bit) bad = 1;
        }
    }
    if (__syncthreads_or(bad) && threadIdx.x == 0) {
        tel_out[cand] = -1;
        atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_ORDER);
    }
}

__global__ __launch_bounds__(256) void check_moves_kernel(const int32_t *moves, int32_t K, int32_t n,
                                                          int64_t *tel_out, int32_t *words)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= K) return;
    const int ty = moves[3 * (size_t)m], i = moves[3 * (size_t)m + 1], j = moves[3 * (size_t)m + 2];
    if ((ty != KVSCHED_MOVE_SWAP && ty != KVSCHED_MOVE_INSERT) || i < 0 || j < 0 || i >= n || j >= n) {
        tel_out[m] = -1;
        atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_MOVE);
    }
}

// One block: index of the least non-negative tel[0..K), lowest index among equals.  With
// with_base, tel[K] is the base order's own latency and becomes the third result.  Fixed
// reduction order, so the result is deterministic.
__global__ __launch_bounds__(1024) void argmin_kernel(const int64_t *tel, int32_t K, int64_t *result_out,
                                                      int32_t with_base)
{
    __shared__ long long sh_tel[16];
    __shared__ int sh_idx[16];
    long long bt = -1;
    int bi = -1;
    for (int m = threadIdx.x; m < K; m += blockDim.x) {
        const long long v = tel[m];
        if (v >= 0 && (bi < 0 || v < bt)) {  // m increases, so ties keep the lower index
            bt = v;
            bi = m;
        }
    }
    // (least latency, then lowest index) is a total order: any reduction tree gives the same winner
    auto take = [&](long long ot, int oi) {
        if (oi >= 0 && (bi < 0 || ot < bt || (ot == bt && oi < bi))) {
            bt = ot;
            bi = oi;
        }
    };
    for (int d = 32; d > 0; d >>= 1) {
        const long long ot = __shfl_xor(bt, d);
        const int oi = __shfl_xor(bi, d);
        take(ot, oi);
    }
    if ((threadIdx.x & 63) == 0) {
        sh_tel[threadIdx.x >> 6] = bt;
        sh_idx[threadIdx.x >> 6] = bi;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        bt = threadIdx.x < 16 ? sh_tel[threadIdx.x] : -1;
        bi = threadIdx.x < 16 ? sh_idx[threadIdx.x] : -1;
        for (int d = 8; d > 0; d >>= 1) {
            const long long ot = __shfl_xor(bt, d);
            const int oi = __shfl_xor(bi, d);
            take(ot, oi);
        }
        if (threadIdx.x == 0) {
            sh_tel[0] = bt;
            sh_idx[0] = bi;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const bool base_ok = !with_base || tel[K] >= 0;  // a faulty base order makes every neighbour faulty
        result_out[0] = base_ok ? sh_idx[0] : -1;
        result_out[1] = (base_ok && sh_idx[0] >= 0) ? sh_tel[0] : -1;
        if (with_base) result_out[2] = tel[K];
    }
}

template <int H, int WPB>
int launch_timeline(const SimParams &p, hipStream_t st)
{
    const unsigned blocks = (unsigned)((p.C + WPB - 1) / WPB);
    if (p.src.orders)
        hipLaunchKernelGGL((timeline_kernel<H, WPB, false>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
    else
        hipLaunchKernelGGL((timeline_kernel<H, WPB, true>), dim3(blocks), dim3(WAVE * WPB), 0, st, p);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

}  // namespace

int kvs_launch_scan_lengths(const int32_t *s, const int32_t *o, int32_t n, int32_t M, int32_t o_bound,
                            int32_t *d_words, hipStream_t st)
{
    hipLaunchKernelGGL(scan_lengths_kernel, dim3(1), dim3(1024), 0, st, s, o, n, M, o_bound, d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_simulate(const SimParams &p, int32_t ring_slots, hipStream_t st)
{
    switch (ring_slots) {
        case 64: return launch_timeline<64, 4>(p, st);
        case 128: return launch_timeline<128, 4>(p, st);
        case 256: return launch_timeline<256, 4>(p, st);
        case 512: return launch_timeline<512, 4>(p, st);
        case 1024: return launch_timeline<1024, 4>(p, st);
        case 2048: return launch_timeline<2048, 4>(p, st);
        case 4096: return launch_timeline<4096, 4>(p, st);
        case 8192: return launch_timeline<8192, 2>(p, st);
        case 16384: return launch_timeline<16384, 1>(p, st);
        default: return KVSCHED_ERANGE;
    }
}

int kvs_launch_check_orders(const int32_t *orders, int32_t C, int32_t n, int64_t *tel_out, int32_t *d_words,
                            hipStream_t st)
{
    const size_t per_wave = (size_t)((n + 31) >> 5) * sizeof(unsigned int);
    if (per_wave > 65536) return KVSCHED_ERANGE;
    if (n >= 16384 && C <= 8192) {  // long rows, not enough of them to fill the chip with a wavefront each
        hipLaunchKernelGGL(check_orders_wide_kernel, dim3((unsigned)C), dim3(1024), per_wave, st, orders, C, n, tel_out,
                           d_words);
    } else if (per_wave * 4 <= 65536) {
        hipLaunchKernelGGL((check_orders_kernel<4>), dim3((unsigned)((C + 3) / 4)), dim3(256), per_wave * 4, st,
                           orders, C, n, tel_out, d_words);
    } else {
        hipLaunchKernelGGL((check_orders_kernel<1>), dim3((unsigned)C), dim3(64), per_wave, st, orders, C, n,
                           tel_out, d_words);
    }
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_check_moves(const int32_t *moves, int32_t K, int32_t n, int64_t *tel_out, int32_t *d_words,
                           hipStream_t st)
{
    hipLaunchKernelGGL(check_moves_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, moves, K, n,
                       tel_out, d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_argmin(const int64_t *tel, int32_t K, int64_t *result_out, int32_t with_base, hipStream_t st)
{
    hipLaunchKernelGGL(argmin_kernel, dim3(1), dim3(1024), 0, st, tel, K, result_out, with_base);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
