// Offline profiling on the device (Section 2.1 Eq. 1, Section 2.2 Eq. 2-4, Alg. 1): the layer-wise
// threshold, the per-token group-argmax counts and the suppression table built from them.
// The two kernels that read the activations are HBM-bandwidth-bound, read-only streams.
#include <mutex>

#include "osc_internal.h"
#include "wave_util.h"

namespace osc {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int PT = 1024;           // threads per workgroup (sixteen wavefronts)
constexpr int PW = PT / 64;
constexpr int P_SEG_CHUNKS = 128;  // 16-byte chunks of one row handled by a wavefront per trip
constexpr int P_SEG_CH = P_SEG_CHUNKS * 8;

// Work split of both streaming kernels: a workgroup owns one 1024-channel column strip `seg` and
// the rows slot*16 + wave, + 16*nslots, ...; two rows are in flight per wavefront and trip, the next
// trip's loads are issued before the current trip is reduced.
struct PLoad {
    u32x4 a0, a1, b0, b1;  // row r: chunks lane, lane+64; row r + rstep: the same
};

__device__ __forceinline__ PLoad profile_load(const uint16_t* __restrict__ X, int64_t ldx, int64_t r,
                                              int64_t rstep, int64_t S, int c0, int nchunk) {
    PLoad p;
    const u32x4 z = {0u, 0u, 0u, 0u};
    p.a0 = p.a1 = p.b0 = p.b1 = z;
    if (r < S) {
        const u32x4* src = reinterpret_cast<const u32x4*>(X + r * ldx);
        if (c0 < nchunk) p.a0 = __builtin_nontemporal_load(src + c0);
        if (c0 + 64 < nchunk) p.a1 = __builtin_nontemporal_load(src + c0 + 64);
    }
    if (r + rstep < S) {
        const u32x4* src = reinterpret_cast<const u32x4*>(X + (r + rstep) * ldx);
        if (c0 < nchunk) p.b0 = __builtin_nontemporal_load(src + c0);
        if (c0 + 64 < nchunk) p.b1 = __builtin_nontemporal_load(src + c0 + 64);
    }
    return p;
}

// ------------------------------------------------------------------------------------------
// Eq. 1, the sum: abs_sum += sum |x|.  Eight magnitudes of a chunk are added as a tree in single
// precision (every input has 8 significant bits, so the tree is off by at most 3 roundings of
// 2^-24), chunks are added in double per lane, lanes and wavefronts in double.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float chunk_abs_sum(u32x4 w) {
    const uint32_t x = w.x, y = w.y, z = w.z, u = w.w;  // scalars first, then the bit casts
    const uint32_t b0 = (x << 16) & 0x7fff0000u, b1 = x & 0x7fff0000u;
    const uint32_t b2 = (y << 16) & 0x7fff0000u, b3 = y & 0x7fff0000u;
    const uint32_t b4 = (z << 16) & 0x7fff0000u, b5 = z & 0x7fff0000u;
    const uint32_t b6 = (u << 16) & 0x7fff0000u, b7 = u & 0x7fff0000u;
    const float e0 = __builtin_bit_cast(float, b0), e1 = __builtin_bit_cast(float, b1);
    const float e2 = __builtin_bit_cast(float, b2), e3 = __builtin_bit_cast(float, b3);
    const float e4 = __builtin_bit_cast(float, b4), e5 = __builtin_bit_cast(float, b5);
    const float e6 = __builtin_bit_cast(float, b6), e7 = __builtin_bit_cast(float, b7);
    return ((e0 + e1) + (e2 + e3)) + ((e4 + e5) + (e6 + e7));
}

__global__ void __launch_bounds__(PT) profile_abs_sum_kernel(const uint16_t* __restrict__ X, int64_t S,
                                                             int H, int64_t ldx, int nseg, int nslots,
                                                             double* __restrict__ abs_sum) {
    __shared__ double part[PW];
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: row and segment arithmetic stays on the scalar unit
    const int seg = blockIdx.x % nseg, slot = blockIdx.x / nseg;
    const int nchunk = H >> 3;
    const int c0 = seg * P_SEG_CHUNKS + lane;
    const int64_t rstep = (int64_t)nslots * PW, rtrip = 2 * rstep;
    double acc = 0.0;
    int64_t r = (int64_t)slot * PW + wave;
    PLoad cur = profile_load(X, ldx, r, rstep, S, c0, nchunk);
    for (; r < S; r += rtrip) {
        const PLoad nxt = profile_load(X, ldx, r + rtrip, rstep, S, c0, nchunk);
        acc += (double)chunk_abs_sum(cur.a0);
        acc += (double)chunk_abs_sum(cur.a1);
        acc += (double)chunk_abs_sum(cur.b0);
        acc += (double)chunk_abs_sum(cur.b1);
        cur = nxt;
    }
#pragma unroll
    for (int o = 32; o; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (t == 0) {
        double s = 0.0;
        for (int i = 0; i < PW; ++i) s += part[i];
        if (s != 0.0) atomicAdd(abs_sum, s);  // one atomic per workgroup: same-address atomics serialise
    }
}

// T = alpha * abs_sum / count, rounded once to single precision.
__global__ void profile_threshold_kernel(const double* __restrict__ abs_sum, double count, double alpha,
                                         float* __restrict__ T) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *T = (float)(alpha * (*abs_sum / count));
}

// ------------------------------------------------------------------------------------------
// Eq. 2 and Eq. 3.  A lane holds 8 channels of a group; a sort key (magnitude bits << 6) |
// (63 - local index) makes "largest magnitude, lowest index among equals" one unsigned maximum:
// three v_max3 in the lane, then DPP exchanges over the 2, 4 or 8 lanes of the group.  The
// group's first lane compares the magnitude with the threshold on bit patterns
// (|x| > T  <=>  bits(|x|) > bits(T) >> 16 for a bf16 x and T >= 0) and bumps the workgroup's
// LDS counter of that channel.  Counters leave once, at the end, as integer atomics on the
// non-zero entries only, so the result does not depend on any ordering.
// ------------------------------------------------------------------------------------------
template <int G>
__device__ __forceinline__ void hist_chunk(u32x4 w, int c, int nchunk, int lane, int tb, int seg_chunk0,
                                           uint32_t* __restrict__ lhist) {
    constexpr int LPG = G / 8;  // lanes per group
    const uint32_t base = 63u - (uint32_t)((lane & (LPG - 1)) * 8);
    const uint32_t k0 = ((w.x & 0x7fffu) << 6) | base;
    const uint32_t k1 = (((w.x >> 16) & 0x7fffu) << 6) | (base - 1u);
    const uint32_t k2 = ((w.y & 0x7fffu) << 6) | (base - 2u);
    const uint32_t k3 = (((w.y >> 16) & 0x7fffu) << 6) | (base - 3u);
    const uint32_t k4 = ((w.z & 0x7fffu) << 6) | (base - 4u);
    const uint32_t k5 = (((w.z >> 16) & 0x7fffu) << 6) | (base - 5u);
    const uint32_t k6 = ((w.w & 0x7fffu) << 6) | (base - 6u);
    const uint32_t k7 = (((w.w >> 16) & 0x7fffu) << 6) | (base - 7u);
    uint32_t k = max(max(max(k0, k1), max(k2, k3)), max(max(k4, k5), max(k6, k7)));
    k = max(k, (uint32_t)__builtin_amdgcn_mov_dpp((int)k, 0xB1, 0xF, 0xF, true));  // lane ^ 1
    if (LPG >= 4) k = max(k, (uint32_t)__builtin_amdgcn_mov_dpp((int)k, 0x4E, 0xF, 0xF, true));   // lane ^ 2
    if (LPG >= 8) k = max(k, (uint32_t)__builtin_amdgcn_mov_dpp((int)k, 0x141, 0xF, 0xF, true));  // 7 - lane in each 8
    if ((lane & (LPG - 1)) == 0 && c < nchunk && (int)(k >> 6) > tb) {
        const int jstar = 63 - (int)(k & 63u);
        atomicAdd(&lhist[(c - seg_chunk0) * 8 + jstar], 1u);
    }
}

template <int G>
__global__ void __launch_bounds__(PT) profile_hist_kernel(const uint16_t* __restrict__ X, int64_t S, int H,
                                                          int64_t ldx, int nseg, int nslots,
                                                          const float* __restrict__ Tptr,
                                                          uint32_t* __restrict__ hist) {
    __shared__ uint32_t lhist[P_SEG_CH];
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: row and segment arithmetic stays on the scalar unit
    const int seg = blockIdx.x % nseg, slot = blockIdx.x / nseg;
    const int nchunk = H >> 3;
    const int sc0 = seg * P_SEG_CHUNKS;
    const int c0 = sc0 + lane;
    const int64_t rstep = (int64_t)nslots * PW, rtrip = 2 * rstep;
    int64_t r = (int64_t)slot * PW + wave;
    PLoad cur = profile_load(X, ldx, r, rstep, S, c0, nchunk);
    // threshold as a bound on magnitude bit patterns: negative T admits everything (zeros too),
    // NaN or infinite T nothing
    const float T = *Tptr;
    const uint32_t tbits = __builtin_bit_cast(uint32_t, T);
    int tb = (int)(tbits >> 16);
    if (tbits & 0x80000000u) tb = -1;
    if ((tbits & 0x7fffffffu) >= 0x7f800000u) tb = 0x7fff;
    for (int i = t; i < P_SEG_CH; i += PT) lhist[i] = 0u;
    __syncthreads();
    for (; r < S; r += rtrip) {
        const PLoad nxt = profile_load(X, ldx, r + rtrip, rstep, S, c0, nchunk);
        hist_chunk<G>(cur.a0, c0, nchunk, lane, tb, sc0, lhist);
        hist_chunk<G>(cur.a1, c0 + 64, nchunk, lane, tb, sc0, lhist);
        if (r + rstep < S) {
            hist_chunk<G>(cur.b0, c0, nchunk, lane, tb, sc0, lhist);
            hist_chunk<G>(cur.b1, c0 + 64, nchunk, lane, tb, sc0, lhist);
        }
        cur = nxt;
    }
    __syncthreads();
    for (int i = t; i < P_SEG_CH; i += PT) {
        const uint32_t v = lhist[i];
        const int ch = seg * P_SEG_CH + i;
        if (v && ch < H) atomicAdd(&hist[ch], v);
    }
}

// ------------------------------------------------------------------------------------------
// Alg. 1's table entry (mode of the candidate set, -1 when empty; the R most frequent indices
// in general) and Eq. 4 with the density.  A wavefront per group at a time with one counter per
// lane; "largest count, lowest index among equals" is a 64-lane
// maximum of the key (count << 6) | (63 - index).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(PT) profile_table_kernel(const uint32_t* __restrict__ hist, int Kg, int G,
                                                           int R, int16_t* __restrict__ table,
                                                           uint32_t* __restrict__ n_total,
                                                           uint32_t* __restrict__ n_hit,
                                                           float* __restrict__ density) {
    const int t = threadIdx.x, lane = t & 63, wave = blockIdx.x * PW + (t >> 6);
    constexpr int TB = 2;  // groups whose counters are fetched together (one memory latency per batch)
    for (int k0 = wave * TB; k0 < Kg; k0 += gridDim.x * PW * TB) {
        uint32_t vb[TB];
#pragma unroll
        for (int b = 0; b < TB; ++b)
            vb[b] = (lane < G && k0 + b < Kg) ? __builtin_nontemporal_load(hist + (int64_t)(k0 + b) * G + lane) : 0u;
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            const int k = k0 + b;
            if (k >= Kg) break;
            const uint32_t v = vb[b];
            const uint64_t total = wave_sum_u64(v);
            uint64_t key = v ? ((uint64_t)v << 6 | (uint64_t)(63 - lane)) : 0ull;
            uint64_t best = wave_max_u64(key);
            const uint32_t top = (uint32_t)(best >> 6);
            const double c = total ? (double)top / (double)total : 0.0;
            if (lane == 0) {
                if (n_total) n_total[k] = (uint32_t)total;
                if (n_hit) n_hit[k] = top;
                if (density) density[k] = (float)c;
            }
            for (int r = 0; r < R; ++r) {
                if (r) best = wave_max_u64(key);
                const int pick = best ? 63 - (int)(best & 63ull) : -1;
                if (lane == 0) table[(int64_t)k * R + r] = (int16_t)pick;
                if (lane == pick) key = 0ull;  // taken
            }
        }
    }
}

// Mean density over the groups with a non-empty candidate set: one workgroup, a thread per group,
// partial sums combined in a fixed order.
__global__ void __launch_bounds__(PT) profile_cbar_kernel(const uint32_t* __restrict__ hist, int Kg, int G,
                                                          float* __restrict__ cbar) {
    __shared__ double dsum[PT];
    __shared__ int dcnt[PT];
    const int t = threadIdx.x;
    double mysum = 0.0;
    int mycnt = 0;
    for (int k = t; k < Kg; k += PT) {
        const uint32_t* h = hist + (int64_t)k * G;
        uint64_t total = 0;
        uint32_t top = 0;
        for (int j = 0; j < G; ++j) {
            const uint32_t v = h[j];
            total += v;
            top = max(top, v);
        }
        if (total) {
            mysum += (double)top / (double)total;
            ++mycnt;
        }
    }
    dsum[t] = mysum;
    dcnt[t] = mycnt;
    __syncthreads();
    for (int o = PT / 2; o; o >>= 1) {
        if (t < o) {
            dsum[t] += dsum[t + o];
            dcnt[t] += dcnt[t + o];
        }
        __syncthreads();
    }
    if (t == 0) *cbar = dcnt[0] ? (float)(dsum[0] / (double)dcnt[0]) : 0.0f;
}

// ---- launchers ---------------------------------------------------------------------------

// Grid of the streaming kernels: nseg column strips x nslots row slots; enough workgroups to keep
// every CU's wavefront slots full (two of sixteen wavefronts per CU), few enough that the atomics
// which end each workgroup (all on the same few addresses, so they serialise) stay off the clock.
static void profile_grid(int64_t S, int64_t H, int* nseg, int* nslots) {
    *nseg = (int)((H + P_SEG_CH - 1) / P_SEG_CH);
    const int64_t want = 512 / *nseg > 0 ? 512 / *nseg : 1;
    const int64_t most = (S + PW - 1) / PW;
    *nslots = (int)(want < most ? want : most);
    if (*nslots < 1) *nslots = 1;
}

int launch_profile_abs_sum(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, double* abs_sum,
                           hipStream_t st) {
    int nseg, nslots;
    profile_grid(S, H, &nseg, &nslots);
    hipLaunchKernelGGL(profile_abs_sum_kernel, dim3(nseg * nslots), dim3(PT), 0, st, X, S, (int)H, ldx, nseg,
                       nslots, abs_sum);
    return check_launch("profile_abs_sum_kernel");
}

int launch_profile_threshold(const double* abs_sum, int64_t count, float alpha, float* T, hipStream_t st) {
    hipLaunchKernelGGL(profile_threshold_kernel, dim3(1), dim3(64), 0, st, abs_sum, (double)count,
                       (double)alpha, T);
    return check_launch("profile_threshold_kernel");
}

int launch_profile_hist(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, int32_t G, const float* T,
                        uint32_t* hist, hipStream_t st) {
    int nseg, nslots;
    profile_grid(S, H, &nseg, &nslots);
    const dim3 grid(nseg * nslots), block(PT);
    if (G == 16)
        hipLaunchKernelGGL(profile_hist_kernel<16>, grid, block, 0, st, X, S, (int)H, ldx, nseg, nslots, T, hist);
    else if (G == 32)
        hipLaunchKernelGGL(profile_hist_kernel<32>, grid, block, 0, st, X, S, (int)H, ldx, nseg, nslots, T, hist);
    else
        hipLaunchKernelGGL(profile_hist_kernel<64>, grid, block, 0, st, X, S, (int)H, ldx, nseg, nslots, T, hist);
    return check_launch("profile_hist_kernel");
}

int launch_profile_table(const uint32_t* hist, int32_t Kg, int32_t G, int32_t R, int16_t* table,
                         uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar, hipStream_t st) {
    if (Kg > 0 && (R > 0 || n_total || n_hit || density)) {
        const int wgs = (Kg + PW * 2 - 1) / (PW * 2);
        hipLaunchKernelGGL(profile_table_kernel, dim3(wgs < 1024 ? wgs : 1024), dim3(PT), 0, st, hist, Kg, G, R,
                           table, n_total, n_hit, density);
        const int rc = check_launch("profile_table_kernel");
        if (rc) return rc;
    }
    if (!cbar) return OSC_OK;
    hipLaunchKernelGGL(profile_cbar_kernel, dim3(1), dim3(PT), 0, st, hist, Kg, G, cbar);
    return check_launch("profile_cbar_kernel");
}

// ---- Alg. 1 in one call: threshold, candidate counts, table -------------------------------------
// Scratch layout (caller's workspace): double abs_sum at 0, float T at 8, uint32 hist[H] at 256.
__global__ void profile_clear_kernel(uint32_t* words, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        words[i] = 0u;
}
__global__ void profile_copy_float_kernel(const float* src, float* dst) { *dst = *src; }

size_t profile_scratch_bytes(int64_t H) { return 256 + (size_t)H * 4; }

int launch_profile_calibrate(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha, int32_t R,
                             int16_t* table, uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar,
                             float* T_out, uint8_t* scratch, hipStream_t st) {
    double* abs_sum = reinterpret_cast<double*>(scratch);
    float* T = reinterpret_cast<float*>(scratch + 8);
    uint32_t* hist = reinterpret_cast<uint32_t*>(scratch + 256);
    // a fill kernel, not a memset: callers may record this call into a graph
    const int64_t words = (int64_t)(profile_scratch_bytes(H) / 4);
    const int64_t wgs = (words + 255) / 256;
    hipLaunchKernelGGL(profile_clear_kernel, dim3((unsigned)(wgs < 1024 ? wgs : 1024)), dim3(256), 0, st,
                       reinterpret_cast<uint32_t*>(scratch), words);
    int rc = check_launch("profile_clear_kernel");
    if (rc) return rc;
    if ((rc = launch_profile_abs_sum(X, S, H, ldx, abs_sum, st))) return rc;
    if ((rc = launch_profile_threshold(abs_sum, S * H, alpha, T, st))) return rc;
    if ((rc = launch_profile_hist(X, S, H, ldx, G, T, hist, st))) return rc;
    if ((rc = launch_profile_table(hist, (int32_t)(H / G), G, R, table, n_total, n_hit, density, cbar, st))) return rc;
    if (T_out) {
        hipLaunchKernelGGL(profile_copy_float_kernel, dim3(1), dim3(1), 0, st, T, T_out);
        rc = check_launch("profile_copy_float_kernel");
    }
    return rc;
}

// ---- the same call for callers that cannot allocate -----------------------------------------------
// The intermediate results live in a file-scope device array instead of a caller's workspace.  In
// host code the array's name is only a handle: its device address is looked up once per device
// (every GPU holds its own copy at its own address) and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[256 + 4 * PROFILE_STATIC_MAX_H];

static uint8_t* static_scratch_address() {
    static std::mutex mu;
    static uint8_t* ptr[MAX_DEVICES];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[dev] = static_cast<uint8_t*>(p);
    }
    return ptr[dev];
}

int launch_profile_calibrate_static(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha,
                                    int32_t R, int16_t* table, uint32_t* n_total, uint32_t* n_hit, float* density,
                                    float* cbar, float* T_out, hipStream_t st) {
    uint8_t* const ptr = static_scratch_address();
    if (!ptr) return fail(OSC_ERR_HIP, "osc_profile_calibrate_static: cannot find the device address of the scratch array");
    return launch_profile_calibrate(X, S, H, ldx, G, alpha, R, table, n_total, n_hit, density, cbar, T_out, ptr, st);
}

}  // namespace osc
