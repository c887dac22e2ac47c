// gfx950 kernels of the DRACO encode/decode path.
//
// Every kernel here is a streaming pass over [node][coordinate] fp32 slabs and
// is bound by HBM bandwidth: one lane owns 4 consecutive floats (one 16-byte
// load per row), a wavefront therefore reads 1 KiB of each row per step, and
// the loop over the P rows runs inside the lane so each input byte is read
// from HBM exactly once.  Workgroups are 256 lanes (4 wavefronts).  There is
// no reuse between workgroups, so the blockIdx -> tile map is the identity.
#include "kernels.hpp"

namespace draco {

namespace {

// Slabs are streamed: every byte is used once, so 16-byte accesses carry the
// non-temporal hint (measured on MI355X: +10% on read-dominated passes).
typedef float vfloat4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4(const float* p) {
    const vfloat4 v = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4(float* p, float4 v) {
    vfloat4 w;
    w.x = v.x;
    w.y = v.y;
    w.z = v.z;
    w.w = v.w;
    __builtin_nontemporal_store(w, reinterpret_cast<vfloat4*>(p));
}

// Guarded load of up to 4 floats; missing ones read as 0.
__device__ __forceinline__ float4 ld4_partial(const float* p, int n) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n > 0) v.x = p[0];
    if (n > 1) v.y = p[1];
    if (n > 2) v.z = p[2];
    if (n > 3) v.w = p[3];
    return v;
}
__device__ __forceinline__ void st4_partial(float* p, float4 v, int n) {
    if (n > 0) p[0] = v.x;
    if (n > 1) p[1] = v.y;
    if (n > 2) p[2] = v.z;
    if (n > 3) p[3] = v.w;
}

__device__ __forceinline__ int clamp4(int64_t n) { return n >= 4 ? 4 : (n <= 0 ? 0 : (int)n); }

// Every workgroup but the last of a launch covers whole 16-byte vectors only;
// the kernels branch ONCE, uniformly, on that, so the common path has no
// per-access bounds checks (FULL) and the ragged tail takes the guarded path.
template <bool FULL>
__device__ __forceinline__ float4 ldx(const float* p, int n) {
    if constexpr (FULL) return ld4(p);
    else return ld4_partial(p, n);
}
template <bool FULL>
__device__ __forceinline__ void stx(float* p, float4 v, int n) {
    if constexpr (FULL) st4(p, v);
    else st4_partial(p, v, n);
}
__device__ __forceinline__ bool block_is_full(int64_t len) {
    return (int64_t)(blockIdx.x + 1) * (kBlock * 4) <= len;
}

}  // namespace

// ===========================================================================
// Repetition code
// ===========================================================================

// E^Rep for all nodes: one pass reads each gradient once, forms each group's
// sum in ascending gradient order and stores it r times.  GU groups are loaded
// before the first is summed, so a lane has GU*R 16-byte loads in flight.
template <int R, int GU, bool FULL>
__device__ __forceinline__ void encode_rep_body(const float* __restrict__ G, int64_t ldg, float* __restrict__ Z,
                                                int64_t ldm, int groups, int64_t d) {
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (!FULL && c0 >= d) return;
    const int n = FULL ? 4 : clamp4(d - c0);
    for (int g0 = 0; g0 < groups; g0 += GU) {
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
    if (block_is_full(d)) encode_rep_body<R, GU, true>(G, ldg, Z, ldm, groups, d);
    else encode_rep_body<R, GU, false>(G, ldg, Z, ldm, groups, d);
}

// Any r (also the one-node form with groups = 1, copies = 1).
__global__ __launch_bounds__(kBlock) void encode_rep_generic_kernel(const float* __restrict__ G, int64_t ldg,
                                                                    float* __restrict__ Z, int64_t ldm,
                                                                    int groups, int r, int copies, int64_t d) {
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (c0 >= d) return;
    const int n = clamp4(d - c0);
    for (int g = 0; g < groups; ++g) {
        const float* src = G + (int64_t)g * r * ldg + c0;
        float4 acc = (n == 4) ? ld4(src) : ld4_partial(src, n);
        for (int i = 1; i < r; ++i) {
            const float4 x = (n == 4) ? ld4(src + (int64_t)i * ldg) : ld4_partial(src + (int64_t)i * ldg, n);
            acc.x += x.x;
            acc.y += x.y;
            acc.z += x.z;
            acc.w += x.w;
        }
        float* dst = Z + (int64_t)g * r * ldm + c0;
        for (int i = 0; i < copies; ++i) {
            if (n == 4) st4(dst + (int64_t)i * ldm, acc);
            else st4_partial(dst + (int64_t)i * ldm, acc, n);
        }
    }
}

// Streaming majority vote (Algorithm 2) on the bit patterns of one coordinate.
template <int R>
__device__ __forceinline__ uint32_t vote(const uint32_t (&v)[R]) {
    uint32_t ma = v[0];
    int counter = 0;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        if (counter == 0) {
            ma = v[i];
            counter = 1;
        } else if (v[i] == ma) {
            ++counter;
        } else {
            --counter;
        }
    }
    return ma;
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
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
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
    if (block_is_full(d)) decode_rep_body<R, GU, true>(Rm, ldm, u, wflags, groups, d);
    else decode_rep_body<R, GU, false>(Rm, ldm, u, wflags, groups, d);
    publish_flags(wflags, flags);
}

// Any r: one coordinate per lane, copies re-read from cache for the count.
__global__ __launch_bounds__(kBlock) void decode_rep_generic_kernel(const float* __restrict__ Rm, int64_t ldm,
                                                                    float* __restrict__ u, uint64_t* __restrict__ flags,
                                                                    int groups, int r, int64_t d) {
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    WaveFlags wflags;
    const bool active = c < d;
    float acc = 0.f;
    for (int g = 0; g < groups; ++g) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(Rm) + (int64_t)g * r * ldm + c;
        uint32_t ma = 0;
        int counter = 0;
        if (active) {
            for (int i = 0; i < r; ++i) {
                const uint32_t v = src[(int64_t)i * ldm];
                if (counter == 0) {
                    ma = v;
                    counter = 1;
                } else if (v == ma) {
                    ++counter;
                } else {
                    --counter;
                }
            }
        }
        for (int i = 0; i < r; ++i) {
            const bool bad = active && src[(int64_t)i * ldm] != ma;
            if (__ballot(bad) != 0ull) wflags.set(g * r + i);
        }
        acc += __uint_as_float(ma);
    }
    if (active) u[c] = acc;
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

// ===========================================================================
// Cyclic code
// ===========================================================================

// acc += (tr + i ti) * (x + i y): one instruction sequence wherever it is used
__device__ __forceinline__ void cmac(double tr, double ti, double x, double y, double& are, double& aim) {
    are = fma(tr, x, are);
    are = fma(-ti, y, are);
    aim = fma(tr, y, aim);
    aim = fma(ti, x, aim);
}

// E^Cyc for all nodes: z_n = sum_{t=0}^{2s} coef[n][t] * g_{(n+t) mod P} with
// coef[n][t] = W[(n+t) mod P][n], on packed complex coordinates in fp64.  A lane
// keeps the window g_n .. g_{n+2s} of its two complex coordinates in registers
// and slides it down the P rows, so every gradient row is read from HBM once;
// rows 0..2s-1, needed again by the last 2s nodes, are parked in LDS (each lane
// reads back only what it wrote: no barrier).  Rows are fetched NB-1 rounds of
// R = 2s+1 ahead of the arithmetic (a ring of NB register buffers).
template <int S, int NB, bool FULL, bool WIDE>
__device__ __forceinline__ void encode_cyc_body(const float* __restrict__ G, int64_t ldg, float* __restrict__ Z,
                                                float* __restrict__ Zlo, int64_t ldm,
                                                const double2* __restrict__ coef, int P, int64_t d,
                                                float4* head /* LDS [2S][kBlock] */) {
    constexpr int R = 2 * S + 1;
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (!FULL && c0 >= mlen) return;
    const int nin = FULL ? 4 : clamp4(d - c0);      // gradient floats that exist (the pad of an odd d reads as 0)
    const int nout = FULL ? 4 : clamp4(mlen - c0);  // message floats to write

    double wre[R][2], wim[R][2];  // window slot = row index mod R

    auto put = [&](int slot, const float4& raw) {
        wre[slot][0] = (double)raw.x;
        wim[slot][0] = (double)raw.y;
        wre[slot][1] = (double)raw.z;
        wim[slot][1] = (double)raw.w;
    };
    // fetch the rows that nodes n0 .. n0+R-1 bring into the window
    auto issue = [&](int n0, float4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int kk = n0 + uu + 2 * S;
            if (n0 + uu < P) {
                if (kk < P) buf[uu] = ldx<FULL>(G + (int64_t)kk * ldg + c0, nin);
                else buf[uu] = head[(kk - P) * kBlock + threadIdx.x];
            }
        }
    };
    auto consume = [&](int n0, const float4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                put((uu + 2 * S) % R, buf[uu]);
                const double2* cn = coef + (int64_t)n * R;
                double are0 = 0.0, aim0 = 0.0, are1 = 0.0, aim1 = 0.0;
#pragma unroll
                for (int t = 0; t < R; ++t) {
                    const int slot = (uu + t) % R;
                    const double cr = cn[t].x, ci = cn[t].y;
                    cmac(cr, ci, wre[slot][0], wim[slot][0], are0, aim0);
                    cmac(cr, ci, wre[slot][1], wim[slot][1], are1, aim1);
                }
                const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                stx<FULL>(Z + (int64_t)n * ldm + c0, hi, nout);
                if constexpr (WIDE) {  // second word of the wide wire: what the first rounding lost
                    const float4 lo = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                  (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                    stx<FULL>(Zlo + (int64_t)n * ldm + c0, lo, nout);
                }
            }
        }
    };

#pragma unroll
    for (int k = 0; k < 2 * S; ++k) {
        const float4 raw = ldx<FULL>(G + (int64_t)k * ldg + c0, nin);
        head[k * kBlock + threadIdx.x] = raw;
        put(k, raw);
    }
    float4 buf[NB][R];
#pragma unroll
    for (int b = 0; b < NB - 1; ++b)
        if (b * R < P) issue(b * R, buf[b]);
    for (int n0 = 0; n0 < P; n0 += NB * R) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int cur = n0 + b * R;
            if (cur < P) {
                const int nxt = cur + (NB - 1) * R;
                if (nxt < P) issue(nxt, buf[(b + NB - 1) % NB]);
                consume(cur, buf[b]);
            }
        }
    }
}

template <int S, int NB, bool WIDE>
__global__ __launch_bounds__(kBlock) void encode_cyc_kernel(const float* __restrict__ G, int64_t ldg,
                                                            float* __restrict__ Z, float* __restrict__ Zlo,
                                                            int64_t ldm, const double2* __restrict__ coef, int P,
                                                            int64_t d) {
    extern __shared__ float4 head[];  // [2S][kBlock]
    if (block_is_full(d)) encode_cyc_body<S, NB, true, WIDE>(G, ldg, Z, Zlo, ldm, coef, P, d, head);
    else encode_cyc_body<S, NB, false, WIDE>(G, ldg, Z, Zlo, ldm, coef, P, d, head);
}

// One node: z = sum_t cn[t] * g_t with cn = this node's row of coef.  With
// wrap_rows == 0, Gn holds only the node's r gradients in assignment order;
// with wrap_rows == P it is the full [P][ldg] slab and row (node+t) mod P is
// used (the all-node path for r > 2*kMaxS+1).  Same operation order as the
// all-node kernel, so results are bit-identical.
__global__ __launch_bounds__(kBlock) void encode_cyc_node_kernel(const float* __restrict__ Gn, int64_t ldg,
                                                                 float* __restrict__ z, float* __restrict__ zlo,
                                                                 const double2* __restrict__ cn, int node, int P,
                                                                 int r, int wrap_rows, int64_t d) {
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (c0 >= mlen) return;
    const int nin = clamp4(d - c0);
    const int nout = clamp4(mlen - c0);
    double are0 = 0.0, aim0 = 0.0, are1 = 0.0, aim1 = 0.0;
    for (int t = 0; t < r; ++t) {
        int k = node + t;
        if (k >= P) k -= P;
        const float* p = Gn + (int64_t)(wrap_rows ? k : t) * ldg + c0;
        const float4 raw = (nin == 4) ? ld4(p) : ld4_partial(p, nin);
        cmac(cn[t].x, cn[t].y, (double)raw.x, (double)raw.y, are0, aim0);
        cmac(cn[t].x, cn[t].y, (double)raw.z, (double)raw.w, are1, aim1);
    }
    const float4 out = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
    if (nout == 4) st4(z + c0, out);
    else st4_partial(z + c0, out, nout);
    if (zlo != nullptr) {
        const float4 lo = make_float4((float)(are0 - (double)out.x), (float)(aim0 - (double)out.y),
                                      (float)(are1 - (double)out.z), (float)(aim1 - (double)out.w));
        if (nout == 4) st4(zlo + c0, lo);
        else st4_partial(zlo + c0, lo, nout);
    }
}

// phi step 1: gamma'_j = sum_i f_i * r_j[i].  A workgroup owns a tile of
// kBlock*kProjectLoads float4 (two complex numbers each) of every row, keeps
// its slice of f in registers, and for each row forms a per-wavefront sum in
// fp64; the four wavefront sums are added in fixed order and stored per tile.
template <bool WIDE>
__global__ __launch_bounds__(kBlock) void cyc_project_kernel(const float* __restrict__ Rm,
                                                             const float* __restrict__ Rlo, int64_t ldm,
                                                             const float* __restrict__ f,
                                                             double2* __restrict__ partial, int P, int64_t d) {
    constexpr int K = kProjectLoads;
    __shared__ double2 wsum[kBlock / 64][kMaxNodes];
    const int64_t h = (d + 1) / 2;                                   // complex numbers per row
    const int64_t q0 = (int64_t)blockIdx.x * (kBlock * K) + threadIdx.x;  // my first float4
    const bool tile_full = ((int64_t)(blockIdx.x + 1) * (kBlock * K)) * 2 <= h;
    double f0[K], f1[K];
    int nflt[K];  // message floats that exist in my k-th float4 (4, 2 or 0)
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t q = q0 + (int64_t)k * kBlock;
        const int64_t c = 2 * q;  // first complex index
        f0[k] = (c < h) ? (double)f[c] : 0.0;
        f1[k] = (c + 1 < h) ? (double)f[c + 1] : 0.0;
        nflt[k] = (c + 1 < h) ? 4 : (c < h ? 2 : 0);
    }
    const int wave = threadIdx.x >> 6;
    for (int j = 0; j < P; ++j) {
        const float* row = Rm + (int64_t)j * ldm + q0 * 4;
        float4 x[K];
        if (tile_full) {
#pragma unroll
            for (int k = 0; k < K; ++k) x[k] = ld4(row + (int64_t)k * kBlock * 4);
        } else {
#pragma unroll
            for (int k = 0; k < K; ++k) x[k] = ld4_partial(row + (int64_t)k * kBlock * 4, nflt[k]);
        }
        double are = 0.0, aim = 0.0;
        if constexpr (WIDE) {  // wire value = hi + lo, exact in fp64
            const float* rowl = Rlo + (int64_t)j * ldm + q0 * 4;
            float4 xl[K];
            if (tile_full) {
#pragma unroll
                for (int k = 0; k < K; ++k) xl[k] = ld4(rowl + (int64_t)k * kBlock * 4);
            } else {
#pragma unroll
                for (int k = 0; k < K; ++k) xl[k] = ld4_partial(rowl + (int64_t)k * kBlock * 4, nflt[k]);
            }
#pragma unroll
            for (int k = 0; k < K; ++k) {
                are = fma(f0[k], (double)x[k].x + (double)xl[k].x, are);
                aim = fma(f0[k], (double)x[k].y + (double)xl[k].y, aim);
                are = fma(f1[k], (double)x[k].z + (double)xl[k].z, are);
                aim = fma(f1[k], (double)x[k].w + (double)xl[k].w, aim);
            }
        } else {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                are = fma(f0[k], (double)x[k].x, are);
                aim = fma(f0[k], (double)x[k].y, aim);
                are = fma(f1[k], (double)x[k].z, are);
                aim = fma(f1[k], (double)x[k].w, aim);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            are += __shfl_xor(are, off);
            aim += __shfl_xor(aim, off);
        }
        if ((threadIdx.x & 63) == 0) wsum[wave][j] = make_double2(are, aim);
    }
    __syncthreads();
    if ((int)threadIdx.x < P) {
        double2 a = wsum[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            a.x += wsum[w][threadIdx.x].x;
            a.y += wsum[w][threadIdx.x].y;
        }
        partial[(int64_t)blockIdx.x * P + threadIdx.x] = a;
    }
}

// gamma[j] = sum over tiles of partial[tile][j], in a fixed order.
__global__ __launch_bounds__(kBlock) void cyc_project_reduce_kernel(const double2* __restrict__ partial,
                                                                    double2* __restrict__ gamma, int P,
                                                                    int64_t tiles) {
    __shared__ double2 sm[kBlock];
    const int j = blockIdx.x;
    double2 a = make_double2(0.0, 0.0);
    for (int64_t t = threadIdx.x; t < tiles; t += kBlock) {
        const double2 p = partial[t * P + j];
        a.x += p.x;
        a.y += p.y;
    }
    sm[threadIdx.x] = a;
    __syncthreads();
    for (int off = kBlock / 2; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off) {
            sm[threadIdx.x].x += sm[threadIdx.x + off].x;
            sm[threadIdx.x].y += sm[threadIdx.x + off].y;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) gamma[j] = sm[0];
}

// u = R_{.,U} b on packed complex messages, unpacked to reals: honest rows in
// ascending node order, fp64 accumulation, one rounding to fp32.
template <bool FULL, bool WIDE>
__device__ __forceinline__ void cyc_recombine_body(const float* __restrict__ Rm, const float* __restrict__ Rlo,
                                                   int64_t ldm,
                                                   const double2* __restrict__ b, const int32_t* __restrict__ idx,
                                                   const int32_t* __restrict__ nu_ptr, float* __restrict__ u,
                                                   int64_t d) {
    constexpr int UN = 8;
    const int nu = *nu_ptr;  // honest nodes; written by the locator (device) or copied in by the host path
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (!FULL && c0 >= d) return;
    const int64_t mlen = 2 * ((d + 1) / 2);
    const int nin = FULL ? 4 : clamp4(mlen - c0);
    const int nout = FULL ? 4 : clamp4(d - c0);
    double are0 = 0.0, aim0 = 0.0, are1 = 0.0, aim1 = 0.0;
    for (int q0 = 0; q0 < nu; q0 += UN) {
        float4 x[UN], xl[WIDE ? UN : 1];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            if (q0 + i < nu) {
                x[i] = ldx<FULL>(Rm + (int64_t)idx[q0 + i] * ldm + c0, nin);
                if constexpr (WIDE) xl[i] = ldx<FULL>(Rlo + (int64_t)idx[q0 + i] * ldm + c0, nin);
            }
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            if (q0 + i < nu) {
                const double br = b[q0 + i].x, bi = b[q0 + i].y;
                if constexpr (WIDE) {
                    cmac(br, bi, (double)x[i].x + (double)xl[i].x, (double)x[i].y + (double)xl[i].y, are0, aim0);
                    cmac(br, bi, (double)x[i].z + (double)xl[i].z, (double)x[i].w + (double)xl[i].w, are1, aim1);
                } else {
                    cmac(br, bi, (double)x[i].x, (double)x[i].y, are0, aim0);
                    cmac(br, bi, (double)x[i].z, (double)x[i].w, are1, aim1);
                }
            }
        }
    }
    stx<FULL>(u + c0, make_float4((float)are0, (float)aim0, (float)are1, (float)aim1), nout);
}

template <bool WIDE>
__global__ __launch_bounds__(kBlock) void cyc_recombine_kernel(const float* __restrict__ Rm,
                                                               const float* __restrict__ Rlo, int64_t ldm,
                                                               const double2* __restrict__ b,
                                                               const int32_t* __restrict__ idx,
                                                               const int32_t* __restrict__ nu,
                                                               float* __restrict__ u, int64_t d) {
    if (block_is_full(d)) cyc_recombine_body<true, WIDE>(Rm, Rlo, ldm, b, idx, nu, u, d);
    else cyc_recombine_body<false, WIDE>(Rm, Rlo, ldm, b, idx, nu, u, d);
}

// Plain copy of a [rows][ld] slab (row_len floats used per row) with the access
// pattern of the encoders: a lane owns one 16-byte column of every row and has
// eight rows in flight.  Calibration kernel for bandwidth figures and for
// scaling hardware byte counters.
__global__ __launch_bounds__(kBlock) void copy_probe_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                            int rows, int64_t row_len, int64_t ld) {
    constexpr int UN = 8;
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (c0 + 4 > row_len) return;
    for (int j0 = 0; j0 < rows; j0 += UN) {
        float4 x[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i)
            if (j0 + i < rows) x[i] = ld4(src + (int64_t)(j0 + i) * ld + c0);
#pragma unroll
        for (int i = 0; i < UN; ++i)
            if (j0 + i < rows) st4(dst + (int64_t)(j0 + i) * ld + c0, x[i]);
    }
}

// ===========================================================================
// Launchers
// ===========================================================================

static inline unsigned grid_for(int64_t units_of_4_floats) {
    return (unsigned)((units_of_4_floats + kBlock - 1) / kBlock);
}

// --- occupancy throttle -----------------------------------------------------
// HBM throughput on MI355X peaks when a CU has roughly 24-48 KiB of loads in
// flight (measured: a [45][25.6M] copy runs at 5.3 TB/s with 32 resident
// wavefronts per CU and at 5.9 TB/s with 4; a read-only pass at 6.1 vs 6.7).
// The streaming kernels therefore ask for more LDS than they use, so that only
// `blocks_per_cu` workgroups fit on a CU at a time.
static size_t lds_per_cu() {
    static const size_t v = [] {
        int dev = 0, val = 0;
        if (hipGetDevice(&dev) != hipSuccess) return (size_t)65536;
        if (hipDeviceGetAttribute(&val, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess || val <= 0)
            return (size_t)65536;
        return (size_t)val;
    }();
    return v;
}

// Dynamic LDS bytes to request so that at most blocks_per_cu workgroups are
// resident per CU (0 = no limit), given the kernel's static LDS use and the
// dynamic bytes it really needs.
static size_t throttle_lds(int blocks_per_cu, size_t static_bytes, size_t needed) {
    if (blocks_per_cu <= 0) return needed;
    size_t per = lds_per_cu() / (size_t)blocks_per_cu;
    per = per / 1024 * 1024;
    const size_t dyn = per > static_bytes ? per - static_bytes : 0;
    return dyn > needed ? dyn : needed;
}

// Opt a kernel in to workgroups with more than 64 KiB of dynamic LDS (once);
// static_bytes is what the kernel declares itself.
template <auto Kernel>
static void allow_large_lds(size_t static_bytes = 0) {
    static const hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)(lds_per_cu() - static_bytes));
    if (e != hipSuccess) (void)hipGetLastError();  // the launch itself reports a request that does not fit
}

// Groups fetched per round (GU0 for r = 1, GU1 for r = 3, one group otherwise):
// keeps r * groups 16-byte loads in flight per lane.
#define DRACO_REP_DISPATCH(KERNEL, GU0, GU1, ...)                                          \
    switch (s) {                                                                           \
        case 0: KERNEL(1, GU0, __VA_ARGS__); break;                                        \
        case 1: KERNEL(3, GU1, __VA_ARGS__); break;                                        \
        case 2: KERNEL(5, 1, __VA_ARGS__); break;                                          \
        case 3: KERNEL(7, 1, __VA_ARGS__); break;                                          \
        case 4: KERNEL(9, 1, __VA_ARGS__); break;                                          \
        case 5: KERNEL(11, 1, __VA_ARGS__); break;                                         \
        case 6: KERNEL(13, 1, __VA_ARGS__); break;                                         \
        case 7: KERNEL(15, 1, __VA_ARGS__); break;                                         \
        default: generic = true;                                                           \
    }

hipError_t launch_encode_rep(const float* G, int64_t ldg, float* Z, int64_t ldm, int P, int s, int64_t d,
                             hipStream_t stream) {
    const int r = 2 * s + 1, groups = P / r;
    const dim3 grid(grid_for((d + 3) / 4)), block(kBlock);
    bool generic = false;
#define DRACO_LAUNCH(R, GU, BPC)                                                                             \
    {                                                                                                        \
        allow_large_lds<encode_rep_kernel<R, GU>>();                                                         \
        hipLaunchKernelGGL((encode_rep_kernel<R, GU>), grid, block, throttle_lds(BPC, 0, 0), stream, G, ldg, \
                           Z, ldm, groups, d);                                                               \
    }
    DRACO_REP_DISPATCH(DRACO_LAUNCH, 8, 2, 1)
#undef DRACO_LAUNCH
    if (generic) hipLaunchKernelGGL(encode_rep_generic_kernel, grid, block, 0, stream, G, ldg, Z, ldm, groups, r, r, d);
    return hipGetLastError();
}

hipError_t launch_encode_rep_node(const float* Gn, int64_t ldg, float* z, int s, int64_t d, hipStream_t stream) {
    const dim3 grid(grid_for((d + 3) / 4)), block(kBlock);
    hipLaunchKernelGGL(encode_rep_generic_kernel, grid, block, 0, stream, Gn, ldg, z, (int64_t)0, 1, 2 * s + 1, 1, d);
    return hipGetLastError();
}

hipError_t launch_decode_rep_vote(const float* R, int64_t ldm, float* u, uint64_t* flags, int P, int s, int64_t d,
                                  hipStream_t stream) {
    const int r = 2 * s + 1, groups = P / r;
    const dim3 block(kBlock);
    const dim3 grid(grid_for((d + 3) / 4));
    bool generic = false;
#define DRACO_LAUNCH(R_, GU, BPC)                                                                               \
    {                                                                                                           \
        allow_large_lds<decode_rep_kernel<R_, GU>>(kMaskWords * sizeof(unsigned long long));                                                           \
        hipLaunchKernelGGL((decode_rep_kernel<R_, GU>), grid, block,                                            \
                           throttle_lds(BPC, kMaskWords * sizeof(unsigned long long), 0), stream, R, ldm, u,    \
                           flags, groups, d);                                                                   \
    }
    DRACO_REP_DISPATCH(DRACO_LAUNCH, 4, 1, 2)
#undef DRACO_LAUNCH
    if (generic) {
        const dim3 g1((unsigned)((d + kBlock - 1) / kBlock));
        hipLaunchKernelGGL(decode_rep_generic_kernel, g1, block, 0, stream, R, ldm, u, flags, groups, r, d);
    }
    return hipGetLastError();
}

hipError_t launch_decode_rep_finish(uint64_t* flags, uint64_t* mask_out, int32_t* status_out, int P, int s,
                                    hipStream_t stream) {
    hipLaunchKernelGGL(decode_rep_finish_kernel, dim3(1), dim3(64), 0, stream, flags, mask_out, status_out, P, s);
    return hipGetLastError();
}

template <int S, int NB>
static void launch_encode_cyc_one(dim3 grid, size_t lds, hipStream_t stream, const float* G, int64_t ldg, float* Z,
                                  float* Zlo, int64_t ldm, const double2* coef, int P, int64_t d) {
    if (Zlo == nullptr) {
        allow_large_lds<encode_cyc_kernel<S, NB, false>>();
        hipLaunchKernelGGL((encode_cyc_kernel<S, NB, false>), grid, dim3(kBlock), lds, stream, G, ldg, Z, Zlo, ldm, coef,
                           P, d);
    } else {
        allow_large_lds<encode_cyc_kernel<S, NB, true>>();
        hipLaunchKernelGGL((encode_cyc_kernel<S, NB, true>), grid, dim3(kBlock), lds, stream, G, ldg, Z, Zlo, ldm, coef,
                           P, d);
    }
}

hipError_t launch_encode_cyc(const float* G, int64_t ldg, float* Z, float* Zlo, int64_t ldm, const double2* coef, int P,
                             int s, int64_t d, hipStream_t stream) {
    const int64_t mlen = 2 * ((d + 1) / 2);
    const dim3 grid(grid_for((mlen + 3) / 4)), block(kBlock);
    const int r = 2 * s + 1;
    // Launch shape from a sweep on MI355X.  Narrow windows on many rows run best with ONE
    // workgroup per CU and rows fetched two rounds ahead (5.7-5.8 TB/s at P = 45 against
    // 5.5 with two workgroups); few rows (short workgroup lifetimes) or wide windows (more
    // fp64 work per byte) need two workgroups per CU to overlap.
    const bool one_per_cu = s <= 3 && P >= 32;
    const size_t lds = throttle_lds(one_per_cu ? 1 : 2, 0, (size_t)2 * s * kBlock * sizeof(float4));
#define DRACO_GO(S, NB) launch_encode_cyc_one<S, NB>(grid, lds, stream, G, ldg, Z, Zlo, ldm, coef, P, d)
    switch (s) {
        case 0: DRACO_GO(0, 3); break;
        case 1: if (one_per_cu) DRACO_GO(1, 3); else DRACO_GO(1, 1); break;
        case 2: if (one_per_cu) DRACO_GO(2, 3); else DRACO_GO(2, 1); break;
        case 3: DRACO_GO(3, 3); break;
        case 4: DRACO_GO(4, 3); break;
        case 5: DRACO_GO(5, 3); break;
        case 6: DRACO_GO(6, 2); break;
        case 7: DRACO_GO(7, 2); break;
        default:
            for (int j = 0; j < P; ++j)
                hipLaunchKernelGGL(encode_cyc_node_kernel, grid, block, 0, stream, G, ldg, Z + (int64_t)j * ldm,
                                   Zlo ? Zlo + (int64_t)j * ldm : nullptr, coef + (int64_t)j * r, j, P, r, P, d);
    }
#undef DRACO_GO
    return hipGetLastError();
}

hipError_t launch_encode_cyc_node(const float* Gn, int64_t ldg, float* z, float* zlo, const double2* coef, int node,
                                  int P, int s, int64_t d, hipStream_t stream) {
    const int64_t mlen = 2 * ((d + 1) / 2);
    const dim3 grid(grid_for((mlen + 3) / 4)), block(kBlock);
    const int r = 2 * s + 1;
    hipLaunchKernelGGL(encode_cyc_node_kernel, grid, block, 0, stream, Gn, ldg, z, zlo, coef + (int64_t)node * r, node,
                       P, r, 0, d);
    return hipGetLastError();
}

int64_t project_tiles(int64_t d) {
    const int64_t h = (d + 1) / 2;
    const int64_t nvec = (h + 1) / 2;
    const int64_t per = (int64_t)kBlock * kProjectLoads;
    return (nvec + per - 1) / per;
}

hipError_t launch_cyc_project(const float* R, const float* Rlo, int64_t ldm, const float* f, double2* partial,
                              double2* gamma, int P, int64_t d, hipStream_t stream) {
    const int64_t tiles = project_tiles(d);
    if (Rlo == nullptr)
        hipLaunchKernelGGL(cyc_project_kernel<false>, dim3((unsigned)tiles), dim3(kBlock), 0, stream, R, Rlo, ldm, f,
                           partial, P, d);
    else
        hipLaunchKernelGGL(cyc_project_kernel<true>, dim3((unsigned)tiles), dim3(kBlock), 0, stream, R, Rlo, ldm, f,
                           partial, P, d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cyc_project_reduce_kernel, dim3((unsigned)P), dim3(kBlock), 0, stream, partial, gamma, P, tiles);
    return hipGetLastError();
}

hipError_t launch_copy_probe(const float* src, float* dst, int rows, int64_t row_len, int64_t ld,
                             hipStream_t stream) {
    allow_large_lds<copy_probe_kernel>();
    hipLaunchKernelGGL(copy_probe_kernel, dim3(grid_for(row_len / 4)), dim3(kBlock), throttle_lds(1, 0, 0), stream, src,
                       dst, rows, row_len, ld);
    return hipGetLastError();
}

hipError_t launch_cyc_recombine(const float* R, const float* Rlo, int64_t ldm, const double2* b, const int32_t* idx,
                                const int32_t* nu, float* u, int64_t d, hipStream_t stream) {
    const dim3 grid(grid_for((d + 3) / 4)), block(kBlock);
    if (Rlo == nullptr) {
        allow_large_lds<cyc_recombine_kernel<false>>();
        hipLaunchKernelGGL(cyc_recombine_kernel<false>, grid, block, throttle_lds(2, 0, 0), stream, R, Rlo, ldm, b, idx,
                           nu, u, d);
    } else {
        allow_large_lds<cyc_recombine_kernel<true>>();
        hipLaunchKernelGGL(cyc_recombine_kernel<true>, grid, block, throttle_lds(2, 0, 0), stream, R, Rlo, ldm, b, idx,
                           nu, u, d);
    }
    return hipGetLastError();
}

}  // namespace draco
