// Routing compaction: from the per-token routing mask to dense lists of routed query rows
// (the "consolidate active queries" preprocessing of the sparse kernel, Sec. 3.2 and App. C
// Alg. 1 step 1; its cost is part of the kernel's time, App. D.1).
//
// Two launches, no host read-back, no spin waits:
//   1. route_count : every workgroup counts the routed rows of its chunk of positions;
//   2. route_write : every workgroup sums the counts of the chunks before it (at most a few
//      hundred integers), then walks its chunk 256 positions at a time; inside a wavefront a
//      row's slot is the pop-count of the ballots of the lanes before it, across wavefronts a
//      4-entry table in LDS.  Rows are written in ascending order, the unused tail gets -1.
#include "common.hpp"

#include <mutex>

// Scratch of l2a_route_compact_static: the per-chunk counts that l2a_route_compact keeps in the
// caller's workspace.  Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress -- never a device address -- so the host side uses static_scratch_ptr().
constexpr int kStaticCounters = 65536;  // 256 KB: (b, KV head, chunk) triples of one call
static __device__ __align__(256) int32_t scratch[kStaticCounters];

namespace l2a {
namespace {

constexpr int kThreads = 256;
// positions per workgroup: 2048, or 256 for sequences so short that 2048 would leave a handful of
// workgroups walking their chunks step by step
__host__ __device__ inline int chunk_positions(int T) { return T <= 16384 ? 256 : 2048; }
constexpr int kMaxG = 16;

struct RouteArgs {
    const uint8_t* mask;
    int32_t* row_idx;
    int32_t* count;
    int32_t* kblk_first_row;
    int32_t* chunk_cnt;
    int B, T, Hq, Hkv, G, Hm, nchunks, nkb, chunk;
};

// mask row of query head (hk, g)
__device__ __forceinline__ const uint8_t* mask_row(const RouteArgs& a, int b, int hk, int g) {
    const int h = hk * a.G + g;
    const int mh = a.Hm == 1 ? 0 : (a.Hm == a.Hq ? h : hk);
    return a.mask + ((size_t)b * a.Hm + mh) * a.T;
}

__device__ __forceinline__ int block_sum(int v, int* lds4) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds4[wave] = v;
    __syncthreads();
    return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

__global__ __launch_bounds__(kThreads) void route_count_kernel(RouteArgs a) {
    __shared__ int lds4[4];
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int b = bh / a.Hkv, hk = bh % a.Hkv;
    const int gdistinct = (a.Hm == a.Hq) ? a.G : 1;  // mask rows that differ inside the group
    const int weight = (a.Hm == a.Hq) ? 1 : a.G;      // rows contributed by one set bit
    int n = 0;
    for (int g = 0; g < gdistinct; ++g) {
        const uint8_t* m = mask_row(a, b, hk, g);
        for (int i = threadIdx.x; i < a.chunk; i += kThreads) {
            const int pos = chunk * a.chunk + i;
            if (pos < a.T && m[pos] != 0) n += weight;
        }
    }
    const int tot = block_sum(n, lds4);
    if (threadIdx.x == 0) a.chunk_cnt[(size_t)bh * a.nchunks + chunk] = tot;
}

__global__ __launch_bounds__(kThreads) void route_write_kernel(RouteArgs a) {
    __shared__ int lds4[4];
    __shared__ int wave_tot[4];
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int b = bh / a.Hkv, hk = bh % a.Hkv;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = a.G;

    // rows before this chunk, and rows in total
    int before = 0, all = 0;
    for (int c = threadIdx.x; c < a.nchunks; c += kThreads) {
        const int v = a.chunk_cnt[(size_t)bh * a.nchunks + c];
        all += v;
        if (c < chunk) before += v;
    }
    before = block_sum(before, lds4);
    all = block_sum(all, lds4);

    int32_t* rows = a.row_idx + (size_t)bh * a.T * G;
    int32_t* first = a.kblk_first_row + (size_t)bh * (a.nkb + 1);
    if (chunk == 0 && threadIdx.x == 0) {
        a.count[bh] = all;
        first[a.nkb] = all;
    }

    const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));  // lanes below this one
    int running = before;
    for (int step = 0; step < a.chunk / kThreads; ++step) {
        const int pos = chunk * a.chunk + step * kThreads + threadIdx.x;
        // bit g of `bits` = d(b, hk*G+g, pos)
        unsigned bits = 0;
        if (pos < a.T) {
            if (a.Hm == a.Hq) {
                for (int g = 0; g < G; ++g) bits |= (mask_row(a, b, hk, g)[pos] != 0 ? 1u : 0u) << g;
            } else {
                bits = mask_row(a, b, hk, 0)[pos] != 0 ? ((1u << G) - 1u) : 0u;
            }
        }
        // rows of the lanes before this one inside the wavefront, and of the whole wavefront
        int excl = 0, wtot = 0;
        for (int g = 0; g < G; ++g) {
            const uint64_t bal = __ballot((bits >> g) & 1u);
            excl += __popcll(bal & lt);
            wtot += __popcll(bal);
        }
        __syncthreads();  // wave_tot of the previous step has been read by everyone
        if (lane == 0) wave_tot[wave] = wtot;
        __syncthreads();
        int wprefix = 0, stot = 0;
        for (int w = 0; w < 4; ++w) {
            const int v = wave_tot[w];
            if (w < wave) wprefix += v;
            stot += v;
        }
        int slot = running + wprefix + excl;
        if (pos < a.T) {
            if ((pos & 63) == 0) first[pos >> 6] = slot;
            for (int g = 0; g < G; ++g)
                if ((bits >> g) & 1u) rows[slot++] = pos * G + g;
        }
        running += stot;
    }

    // unused tail: this workgroup owns slots [chunk * a.chunk * G, (chunk + 1) * a.chunk * G)
    const long long lo = (long long)chunk * a.chunk * G;
    long long hi = lo + (long long)a.chunk * G;
    const long long cap = (long long)a.T * G;
    if (hi > cap) hi = cap;
    for (long long s = lo + threadIdx.x; s < hi; s += kThreads)
        if (s >= all) rows[s] = -1;
}

}  // namespace

size_t route_workspace_bytes(const l2a_params& p) {
    const size_t chunk = chunk_positions(p.T);
    const size_t nchunks = ((size_t)p.T + chunk - 1) / chunk;
    return sizeof(int32_t) * nchunks * (size_t)p.B * (size_t)p.Hkv;
}

// Device address of `scratch` on the current device, looked up once per device.
static int32_t* static_scratch_ptr() {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static int32_t* ptr[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[dev] = (int32_t*)p;
    }
    return ptr[dev];
}

int route_compact_static(const l2a_params& p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                         int32_t* kblk_first_row, hipStream_t st) {
    if (route_workspace_bytes(p) > sizeof(int32_t) * (size_t)kStaticCounters) return L2A_ERR_STATIC_LIMIT;
    int32_t* ws = static_scratch_ptr();
    if (!ws) return L2A_ERR_LAUNCH;
    // every counter the second kernel reads is written by the first: nothing has to start at zero
    return route_compact(p, mask, row_idx, count, kblk_first_row, ws, st);
}

int route_compact(const l2a_params& p, const uint8_t* mask, int32_t* row_idx, int32_t* count,
                  int32_t* kblk_first_row, void* ws, hipStream_t st) {
    RouteArgs a;
    a.mask = mask;
    a.row_idx = row_idx;
    a.count = count;
    a.kblk_first_row = kblk_first_row;
    a.chunk_cnt = (int32_t*)ws;
    a.B = p.B; a.T = p.T; a.Hq = p.Hq; a.Hkv = p.Hkv; a.G = p.Hq / p.Hkv; a.Hm = p.mask_heads;
    a.chunk = chunk_positions(p.T);
    a.nchunks = (p.T + a.chunk - 1) / a.chunk;
    a.nkb = (p.T + 63) / 64;
    if (a.G > kMaxG) return L2A_ERR_UNSUPPORTED;
    const dim3 grid(a.nchunks, p.B * p.Hkv);
    {
        KernelTimer kt("route_count", st);
        hipLaunchKernelGGL(route_count_kernel, grid, dim3(kThreads), 0, st, a);
    }
    {
        KernelTimer kt("route_write", st);
        hipLaunchKernelGGL(route_write_kernel, grid, dim3(kThreads), 0, st, a);
    }
    return launch_status();
}

}  // namespace l2a
