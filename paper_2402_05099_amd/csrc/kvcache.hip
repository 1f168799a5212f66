// KV-cache update of a decode step (Sec. 2.2: the cache holds the keys and values of all earlier tokens and every
// step adds the newest token's; Sec. 3.5: suffix lengths change from step to step while the launch sequence stays
// the same, so lengths live on the device and are advanced there).  Pure data movement: one workgroup per sequence
// copies the nq new K and V rows behind the sequence's last suffix row, then its first thread advances the length.
#include "hg_internal.h"

namespace hg {

__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a) {
    const int b = blockIdx.x;
    const int len = a.lengths[b];          // every thread reads the old length before thread 0 replaces it
    __syncthreads();
    const int room = a.capacity - len;
    const int take = len < 0 ? 0 : room < a.nq ? (room > 0 ? room : 0) : a.nq;   // rows that fit below the capacity
    const int vec = a.row_elems / 8;       // 16-byte groups per row (Hkv * D is a multiple of 64)
    for (int i = threadIdx.x; i < take * vec; i += 256) {
        const int t = i / vec, c = i - t * vec;
        const int j = len + t;             // suffix row that token t becomes
        int64_t row;
        if (a.pg.table) {
            int page = a.pg.table[(int64_t)b * a.pg.stride + (j >> a.pg.shift)];
            page = min(max(page, 0), a.pg.n_pages - 1);
            row = ((int64_t)page << a.pg.shift) + (j & ((1 << a.pg.shift) - 1));
        } else {
            row = (int64_t)a.offsets[b] + j;
        }
        const int64_t src = ((int64_t)b * a.nq + t) * vec + c;
        const int64_t dst = row * vec + c;
        reinterpret_cast<uint4*>(a.Ks)[dst] = reinterpret_cast<const uint4*>(a.Knew)[src];
        reinterpret_cast<uint4*>(a.Vs)[dst] = reinterpret_cast<const uint4*>(a.Vnew)[src];
    }
    if (threadIdx.x == 0 && take > 0) a.lengths[b] = len + take;
}

hipError_t launch_kv_append(const AppendArgs& a, hipStream_t s) {
    if (a.B == 0) return hipSuccess;
    kv_append_kernel<<<(unsigned)a.B, 256, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace hg
