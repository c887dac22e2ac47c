// Repetition code (Sec. 3, "Fractional Repetition Code"): encoder E^Rep and the
// majority-vote decoder D^Rep with the streaming vote of Algorithm 2.
#include "device_util.hpp"

#include <mutex>

namespace draco {

// ===========================================================================
// Repetition code
// ===========================================================================

// E^Rep for all nodes: one pass reads each gradient once, forms each group's
// sum in ascending gradient order and stores it r times.  A workgroup handles
// one column tile (blockIdx.x) of GU consecutive groups (blockIdx.y) and ends:
// with tiles varying fastest across the grid, the whole chip streams the same
// few rows at a time, which HBM serves measurably faster (6.3-6.6 TB/s for a
// copy of this shape) than workgroups that each walk down all P rows (5.9).
// The GU groups are loaded before the first is summed: GU*R 16-byte loads in
// flight per lane.
template <int R, int GU, bool FULL>
__device__ __forceinline__ void encode_rep_body(const float* __restrict__ G, int64_t ldg, float* __restrict__ Z,
                                                int64_t ldm, int groups, int64_t d) {
    const int64_t c0 = lane_column<kSpreadEncodeRep>();
    if (!FULL && c0 >= d) return;
    const int n = FULL ? 4 : clamp4(d - c0);
    {
        const int g0 = (int)blockIdx.y * GU;
        float4 x[GU][R];
#pragma unroll
        for (int a = 0; a < GU; ++a) {
            if (g0 + a < groups) {
                const float* src = G + (int64_t)(g0 + a) * R * ldg + c0;
#pragma unroll
                for (int i = 0; i < R; ++i) x[a][i] = ldx<FULL>(src + (int64_t)i * ldg, n);
            }
        }
#pragma unroll
        for (int a = 0; a < GU; ++a) {
            if (g0 + a < groups) {
                float4 acc = x[a][0];
#pragma unroll
                for (int i = 1; i < R; ++i) {
                    acc.x += x[a][i].x;
                    acc.y += x[a][i].y;
                    acc.z += x[a][i].z;
                    acc.w += x[a][i].w;
                }
                float* dst = Z + (int64_t)(g0 + a) * R * ldm + c0;
#pragma unroll
                for (int i = 0; i < R; ++i) stx<FULL>(dst + (int64_t)i * ldm, acc, n);
            }
        }
    }
}

template <int R, int GU>
__global__ __launch_bounds__(kBlock) void encode_rep_kernel(const float* __restrict__ G, int64_t ldg,
                                                            float* __restrict__ Z, int64_t ldm,
                                                            int groups, int64_t d) {
    if (block_is_full<kSpreadEncodeRep>(d)) encode_rep_body<R, GU, true>(G, ldg, Z, ldm, groups, d);
    else encode_rep_body<R, GU, false>(G, ldg, Z, ldm, groups, d);
}

// Any number of rows per group (also the one-node form with groups = 1, copies = 1, and
// the B > P form where a group sums its r*(B/P) consecutive per-sample rows): rows are
// added in ascending order, eight fetched at a time.
template <bool FULL>
__device__ __forceinline__ void encode_rep_generic_body(const float* __restrict__ G, int64_t ldg,
                                                        float* __restrict__ Z, int64_t ldm, int groups, int rows,
                                                        int copies, int64_t d) {
    constexpr int UN = 8;
    const int64_t c0 = lane_column<kSpreadEncodeRep>();
    if (!FULL && c0 >= d) return;
    const int n = FULL ? 4 : clamp4(d - c0);
    {
        const int g = (int)blockIdx.y;   // one group per workgroup (grid.y = groups)
        if (g >= groups) return;
        const float* src = G + (int64_t)g * rows * ldg + c0;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        int i0 = 0;
        for (; i0 + UN <= rows; i0 += UN) {   // whole rounds: no per-row checks
            float4 x[UN];
#pragma unroll
            for (int i = 0; i < UN; ++i) x[i] = ldx<FULL>(src + (int64_t)(i0 + i) * ldg, n);
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                acc.x += x[i].x;
                acc.y += x[i].y;
                acc.z += x[i].z;
                acc.w += x[i].w;
            }
        }
        for (; i0 < rows; ++i0) {
            const float4 x = ldx<FULL>(src + (int64_t)i0 * ldg, n);
            acc.x += x.x;
            acc.y += x.y;
            acc.z += x.z;
            acc.w += x.w;
        }
        float* dst = Z + (int64_t)g * copies * ldm + c0;
        for (int i = 0; i < copies; ++i) stx<FULL>(dst + (int64_t)i * ldm, acc, n);
    }
}

__global__ __launch_bounds__(kBlock) void encode_rep_generic_kernel(const float* __restrict__ G, int64_t ldg,
                                                                    float* __restrict__ Z, int64_t ldm,
                                                                    int groups, int rows, int copies, int64_t d) {
    if (block_is_full<kSpreadEncodeRep>(d)) encode_rep_generic_body<true>(G, ldg, Z, ldm, groups, rows, copies, d);
    else encode_rep_generic_body<false>(G, ldg, Z, ldm, groups, rows, copies, d);
}

// Majority candidate among R bit patterns of one coordinate (the streaming vote of
// Algorithm 2): one candidate and its lead over everything else seen so far, updated with
// selects only.  A copy that agrees raises the lead, one that differs lowers it, and when
// the lead is used up the next copy takes over as candidate.  If some pattern is held by
// more than half of the copies it is the result.
__device__ __forceinline__ void vote_step(uint32_t copy, uint32_t& candidate, int& lead) {
    const bool vacant = lead == 0;
    const int delta = (copy == candidate) ? 1 : -1;
    candidate = vacant ? copy : candidate;
    lead = vacant ? 1 : lead + delta;
}
template <int R>
__device__ __forceinline__ uint32_t vote(const uint32_t (&v)[R]) {
    uint32_t candidate = v[0];
    int lead = 1;
#pragma unroll
    for (int i = 1; i < R; ++i) vote_step(v[i], candidate, lead);
    return candidate;
}

// Node flags of one wavefront (wavefront-uniform values, kept in scalar registers).
struct WaveFlags {
    uint64_t w[kMaskWords] = {0, 0, 0, 0};
    __device__ __forceinline__ void set(int node) {
        const uint64_t bit = 1ull << (node & 63);
        const int word = node >> 6;
        if (word == 0) w[0] |= bit;
        else if (word == 1) w[1] |= bit;
        else if (word == 2) w[2] |= bit;
        else w[3] |= bit;
    }
};
static_assert(kMaskWords == 4, "WaveFlags::set spells out four words");

// OR the wavefront-uniform flag words of the four wavefronts of a workgroup
// into the global flag words, touching global memory only for bits that are
// not set there yet.
__device__ __forceinline__ void publish_flags(const WaveFlags& wf, uint64_t* __restrict__ flags) {
    __shared__ unsigned long long sflags[kMaskWords];
    if (threadIdx.x < kMaskWords) sflags[threadIdx.x] = 0ull;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        if (wf.w[0]) atomicOr(&sflags[0], (unsigned long long)wf.w[0]);
        if (wf.w[1]) atomicOr(&sflags[1], (unsigned long long)wf.w[1]);
        if (wf.w[2]) atomicOr(&sflags[2], (unsigned long long)wf.w[2]);
        if (wf.w[3]) atomicOr(&sflags[3], (unsigned long long)wf.w[3]);
    }
    __syncthreads();
    if (threadIdx.x < kMaskWords) {
        const unsigned long long mine = sflags[threadIdx.x];
        if (mine) {
            unsigned long long* dst = reinterpret_cast<unsigned long long*>(flags) + threadIdx.x;
            const unsigned long long cur = __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (mine & ~cur) atomicOr(dst, mine);
        }
    }
}

// Vote of one group held in registers: returns the winner of each of the
// lane's four coordinates and ORs the flags of differing nodes (wavefront-
// uniform) into wflags.  Honest groups take the fast path: all copies equal,
// decided for the whole wavefront by one ballot.
template <int R>
__device__ __forceinline__ uint4 vote_group(const uint4 (&x)[R], int first_node, WaveFlags& wflags) {
    uint32_t differ = 0;
#pragma unroll
    for (int i = 1; i < R; ++i)
        differ |= (x[i].x ^ x[0].x) | (x[i].y ^ x[0].y) | (x[i].z ^ x[0].z) | (x[i].w ^ x[0].w);
    uint4 win = x[0];
    if (__ballot(differ != 0) != 0ull) {   // some lane of the wavefront saw a disagreement in this group
        uint32_t bad = 0;                  // bit i: copy i differs from the vote in one of my coordinates
        if (differ != 0) {
            uint32_t v[R];
#pragma unroll
            for (int i = 0; i < R; ++i) v[i] = x[i].x;
            win.x = vote<R>(v);
#pragma unroll
            for (int i = 0; i < R; ++i) bad |= (uint32_t)(v[i] != win.x) << i;
#pragma unroll
            for (int i = 0; i < R; ++i) v[i] = x[i].y;
            win.y = vote<R>(v);
#pragma unroll
            for (int i = 0; i < R; ++i) bad |= (uint32_t)(v[i] != win.y) << i;
#pragma unroll
            for (int i = 0; i < R; ++i) v[i] = x[i].z;
            win.z = vote<R>(v);
#pragma unroll
            for (int i = 0; i < R; ++i) bad |= (uint32_t)(v[i] != win.z) << i;
#pragma unroll
            for (int i = 0; i < R; ++i) v[i] = x[i].w;
            win.w = vote<R>(v);
#pragma unroll
            for (int i = 0; i < R; ++i) bad |= (uint32_t)(v[i] != win.w) << i;
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            if (__ballot((bad >> i) & 1u) != 0ull) wflags.set(first_node + i);
        }
    }
    return win;
}

// D^Rep: per coordinate and group, the vote over the r copies; winners are
// summed over groups in ascending order; a node is flagged when any of its
// coordinates differs from the winner.  GU groups are loaded before the first
// is voted on (GU*R 16-byte loads in flight per lane).
template <int R, int GU, bool FULL>
__device__ __forceinline__ void decode_rep_body(const float* __restrict__ Rm, int64_t ldm, float* __restrict__ u,
                                                WaveFlags& wflags, int groups, int64_t d) {
    const int64_t c0 = lane_column<kSpreadVote>();
    const bool active = FULL || c0 < d;
    const int n = FULL ? 4 : (active ? clamp4(d - c0) : 0);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int g0 = 0; g0 < groups; g0 += GU) {
        uint4 x[GU][R];
#pragma unroll
        for (int a = 0; a < GU; ++a) {
            if (g0 + a < groups) {
                const float* src = Rm + (int64_t)(g0 + a) * R * ldm + c0;
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);   // lanes past the end vote on zeros
                    if (active) t = ldx<FULL>(src + (int64_t)i * ldm, n);
                    x[a][i] = make_uint4(__float_as_uint(t.x), __float_as_uint(t.y), __float_as_uint(t.z),
                                         __float_as_uint(t.w));
                }
            }
        }
#pragma unroll
        for (int a = 0; a < GU; ++a) {
            if (g0 + a < groups) {
                const uint4 win = vote_group<R>(x[a], (g0 + a) * R, wflags);
                acc.x += __uint_as_float(win.x);
                acc.y += __uint_as_float(win.y);
                acc.z += __uint_as_float(win.z);
                acc.w += __uint_as_float(win.w);
            }
        }
    }
    if (active) stx<FULL>(u + c0, acc, n);
}

template <int R, int GU>
__global__ __launch_bounds__(kBlock) void decode_rep_kernel(const float* __restrict__ Rm, int64_t ldm,
                                                            float* __restrict__ u, uint64_t* __restrict__ flags,
                                                            int groups, int64_t d) {
    WaveFlags wflags;
    if (block_is_full<kSpreadVote>(d)) decode_rep_body<R, GU, true>(Rm, ldm, u, wflags, groups, d);
    else decode_rep_body<R, GU, false>(Rm, ldm, u, wflags, groups, d);
    publish_flags(wflags, flags);
}

// Any r: the copies of a group stream through the vote's two words of state per
// coordinate (candidate, lead), eight rows in flight, so every message byte is read
// once.  Only where some lane of the wavefront saw a copy differ from the first one is the
// group read again, to flag the nodes that differ from the winner.
template <bool FULL>
__device__ __forceinline__ void decode_rep_stream_body(const float* __restrict__ Rm, int64_t ldm,
                                                       float* __restrict__ u, WaveFlags& wflags, int groups,
                                                       int r, int64_t d) {
    constexpr int UN = 8;
    const int64_t c0 = lane_column<kSpreadVote>();
    const bool active = FULL || c0 < d;
    const int n = FULL ? 4 : (active ? clamp4(d - c0) : 0);
    auto fetch = [&](const float* p) -> uint4 {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);   // lanes past the end vote on zeros
        if (active) t = ldx<FULL>(p, n);
        return make_uint4(__float_as_uint(t.x), __float_as_uint(t.y), __float_as_uint(t.z), __float_as_uint(t.w));
    };
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int g = 0; g < groups; ++g) {
        const float* src = Rm + (int64_t)g * r * ldm + c0;
        uint4 ma = make_uint4(0u, 0u, 0u, 0u), first = ma;   // ma: the four coordinates' candidates
        int cx = 0, cy = 0, cz = 0, cw = 0;                   // their leads (0: no candidate yet)
        uint32_t differ = 0;
        for (int i0 = 0; i0 < r; i0 += UN) {
            uint4 x[UN];
#pragma unroll
            for (int i = 0; i < UN; ++i)
                if (i0 + i < r) x[i] = fetch(src + (int64_t)(i0 + i) * ldm);
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                if (i0 + i < r) {
                    if (i0 + i == 0) first = x[i];
                    differ |= (x[i].x ^ first.x) | (x[i].y ^ first.y) | (x[i].z ^ first.z) | (x[i].w ^ first.w);
                    vote_step(x[i].x, ma.x, cx);
                    vote_step(x[i].y, ma.y, cy);
                    vote_step(x[i].z, ma.z, cz);
                    vote_step(x[i].w, ma.w, cw);
                }
            }
        }
        if (__ballot(differ != 0) != 0ull) {
            for (int i = 0; i < r; ++i) {
                const uint4 x = fetch(src + (int64_t)i * ldm);
                const bool bad = (x.x != ma.x) | (x.y != ma.y) | (x.z != ma.z) | (x.w != ma.w);
                if (__ballot(bad) != 0ull) wflags.set(g * r + i);
            }
        }
        acc.x += __uint_as_float(ma.x);
        acc.y += __uint_as_float(ma.y);
        acc.z += __uint_as_float(ma.z);
        acc.w += __uint_as_float(ma.w);
    }
    if (active) stx<FULL>(u + c0, acc, n);
}

__global__ __launch_bounds__(kBlock) void decode_rep_generic_kernel(const float* __restrict__ Rm, int64_t ldm,
                                                                    float* __restrict__ u, uint64_t* __restrict__ flags,
                                                                    int groups, int r, int64_t d) {
    WaveFlags wflags;
    if (block_is_full<kSpreadVote>(d)) decode_rep_stream_body<true>(Rm, ldm, u, wflags, groups, r, d);
    else decode_rep_stream_body<false>(Rm, ldm, u, wflags, groups, r, d);
    publish_flags(wflags, flags);
}

__global__ void decode_rep_finish_kernel(uint64_t* __restrict__ flags, uint64_t* __restrict__ mask_out,
                                         int32_t* __restrict__ status_out, int P, int s) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int r = 2 * s + 1;
    int status = 0;
    for (int g = 0; g < P / r; ++g) {
        int cnt = 0;
        for (int i = 0; i < r; ++i) {
            const int node = g * r + i;
            cnt += (int)((flags[node >> 6] >> (node & 63)) & 1ull);
        }
        if (cnt > s) status = 1;  // DRACO_NO_MAJORITY
    }
    for (int w = 0; w < (P + 63) / 64; ++w) mask_out[w] = flags[w];
    for (int w = 0; w < kMaskWords; ++w) flags[w] = 0;
    *status_out = status;
}


// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------

// Groups fetched per round (GU0 for r = 1, GU1 for r = 3, GU2 for r = 5, one group otherwise)
// and workgroups per CU (BPC2 for r = 5, BPC otherwise):
// keeps r * groups 16-byte loads in flight per lane.
#define DRACO_REP_DISPATCH(KERNEL, GU0, GU1, GU2, BPC, BPC2)                                          \
    switch (s) {                                                                           \
        case 0: KERNEL(1, GU0, BPC); break;                                        \
        case 1: KERNEL(3, GU1, BPC); break;                                        \
        case 2: KERNEL(5, GU2, BPC2); break;                                          \
        case 3: KERNEL(7, 1, BPC); break;                                          \
        case 4: KERNEL(9, 1, BPC); break;                                          \
        case 5: KERNEL(11, 1, BPC); break;                                         \
        case 6: KERNEL(13, 1, BPC); break;                                         \
        case 7: KERNEL(15, 1, BPC); break;                                         \
        default: generic = true;                                                           \
    }

hipError_t launch_encode_rep(const float* G, int64_t ldg, float* Z, int64_t ldm, int P, int s, int64_t d,
                             hipStream_t stream) {
    const int r = 2 * s + 1, groups = P / r;
    const unsigned tiles = grid_cols<kSpreadEncodeRep>(d);
    const dim3 block(kBlock);
    bool generic = false;
#define DRACO_LAUNCH(R, GU, BPC)                                                                             \
    {                                                                                                        \
        allow_large_lds<encode_rep_kernel<R, GU>>();                                                         \
        hipLaunchKernelGGL((encode_rep_kernel<R, GU>), dim3(tiles, (unsigned)((groups + GU - 1) / GU)),      \
                           block, throttle_lds(BPC, 0, 0), stream, G, ldg, Z, ldm, groups, d);               \
    }
    DRACO_REP_DISPATCH(DRACO_LAUNCH, 8, 2, 1, 1, 2)
#undef DRACO_LAUNCH
    if (generic) {
        allow_large_lds<encode_rep_generic_kernel>();
        hipLaunchKernelGGL(encode_rep_generic_kernel, dim3(tiles, (unsigned)groups), block, throttle_lds(2, 0, 0),
                           stream, G, ldg, Z, ldm, groups, r, r, d);
    }
    return hipGetLastError();
}

hipError_t launch_encode_rep_samples(const float* G, int64_t ldg, int m, float* Z, int64_t ldm, int P, int s, int64_t d,
                                     hipStream_t stream) {
    const int r = 2 * s + 1, groups = P / r;
    const dim3 grid(grid_cols<kSpreadEncodeRep>(d), (unsigned)groups), block(kBlock);
    allow_large_lds<encode_rep_generic_kernel>();
    hipLaunchKernelGGL(encode_rep_generic_kernel, grid, block, throttle_lds(2, 0, 0), stream, G, ldg, Z, ldm, groups,
                       r * m, r, d);
    return hipGetLastError();
}

hipError_t launch_encode_rep_node(const float* Gn, int64_t ldg, float* z, int s, int64_t d, hipStream_t stream) {
    const dim3 grid(grid_cols<kSpreadEncodeRep>(d)), block(kBlock);
    hipLaunchKernelGGL(encode_rep_generic_kernel, grid, block, 0, stream, Gn, ldg, z, (int64_t)0, 1, 2 * s + 1, 1, d);
    return hipGetLastError();
}

hipError_t launch_decode_rep_vote(const float* R, int64_t ldm, float* u, uint64_t* flags, int P, int s, int64_t d,
                                  hipStream_t stream) {
    const int r = 2 * s + 1, groups = P / r;
    const dim3 block(kBlock);
    const dim3 grid(grid_cols<kSpreadVote>(d));
    bool generic = false;
#define DRACO_LAUNCH(R_, GU, BPC)                                                                               \
    {                                                                                                           \
        allow_large_lds<decode_rep_kernel<R_, GU>>(kMaskWords * sizeof(unsigned long long));                                                           \
        hipLaunchKernelGGL((decode_rep_kernel<R_, GU>), grid, block,                                            \
                           throttle_lds(BPC, kMaskWords * sizeof(unsigned long long), 0), stream, R, ldm, u,    \
                           flags, groups, d);                                                                   \
    }
    // the vote over r = 5 copies is the one shape that runs faster with four workgroups per CU
    // (6.4 against 6.25 TB/s; every other r loses 4-5 % there)
    DRACO_REP_DISPATCH(DRACO_LAUNCH, 4, 1, 1, 2, 4)
#undef DRACO_LAUNCH
    if (generic) {
        allow_large_lds<decode_rep_generic_kernel>(kMaskWords * sizeof(unsigned long long));
        hipLaunchKernelGGL(decode_rep_generic_kernel, grid, block,
                           throttle_lds(2, kMaskWords * sizeof(unsigned long long), 0), stream, R, ldm, u, flags,
                           groups, r, d);
    }
    return hipGetLastError();
}

hipError_t launch_decode_rep_finish(uint64_t* flags, uint64_t* mask_out, int32_t* status_out, int P, int s,
                                    hipStream_t stream) {
    hipLaunchKernelGGL(decode_rep_finish_kernel, dim3(1), dim3(64), 0, stream, flags, mask_out, status_out, P, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// D^Rep without any allocation: the node-flag words live in a device array that is part of
// the loaded code object, one copy per GPU, kept until the process ends.
// ---------------------------------------------------------------------------
namespace {

// Node flags of the allocation-free decoder: kMaskWords 64-bit words (one bit per node,
// kMaxNodes nodes at most).  In host code this name is only a handle for
// hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) unsigned long long scratch[kMaskWords];

constexpr int kMaxDevices = 64;
uint64_t* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, resolved once
std::mutex g_scratch_mutex;

__global__ void clear_flags_kernel(uint64_t* __restrict__ flags) {
    if (blockIdx.x == 0 && threadIdx.x < kMaskWords) flags[threadIdx.x] = 0;
}

// Address of the current device's copy of `scratch` (resolved on the first call per device).
hipError_t static_flags(uint64_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<uint64_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

hipError_t launch_decode_rep_static(const float* R, int64_t ldm, float* u, uint64_t* mask_out, int32_t* status_out,
                                    int P, int s, int64_t d, hipStream_t stream) {
    uint64_t* flags = nullptr;
    hipError_t e = static_flags(&flags);
    if (e != hipSuccess) return e;
    // the array keeps what the last call left (zero after a call that ran to its end); a fill
    // kernel, not a memset, so that the sequence can be captured in a HIP graph
    hipLaunchKernelGGL(clear_flags_kernel, dim3(1), dim3(64), 0, stream, flags);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_decode_rep_vote(R, ldm, u, flags, P, s, d, stream);
    if (e != hipSuccess) return e;
    return launch_decode_rep_finish(flags, mask_out, status_out, P, s, stream);
}


}  // namespace draco
