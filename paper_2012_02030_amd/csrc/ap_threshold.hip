// Layer-wise percentile threshold and pruning mask (Section 3.2, paragraph before Eq. (2), and
// Eq. (2)).
//
// tau is the order statistic of rank floor(p * N) among the N participating entries of the mean
// maps of all heads of a layer.  It is found exactly, by radix selection over the entries' bit
// patterns, in two sweeps over the maps:
//
//   sweep 1  radix_hist_kernel<0>: histogram of the top 15 key bits (32768 bins in LDS);
//            radix_select_kernel<0> picks the bin that holds the wanted rank.  That bin is a
//            value interval about 1 % wide and usually holds well under a million entries.
//   sweep 2  mask_collect_kernel: every entry above the bin is kept, every entry below it is
//            pruned, and the entries inside it (the candidates) are copied out.
//   then     candidate_select_kernel finds tau among the candidates (their remaining 17 bits) and
//            candidate_fixup_kernel writes their mask bytes.
//
// If the bin holds more candidates than the workspace has room for (massive ties), levels 1
// and 2 of the histogram/select pair fix 15 and then 2 more bits with a sweep each before the
// mask sweep; otherwise those launches return at once.  Which path runs is decided on the
// device, so the call never synchronises with the host.
//
// Float bit patterns are mapped to unsigned keys whose integer order is the numeric order
// (sign bit flipped for non-negative values, all bits flipped for negative ones; -0 counts as +0).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

constexpr int kBins = 32768;                 // 15-bit digit
constexpr uint32_t kCap = 1u << 20;          // candidates the workspace can hold
constexpr int kThreads = 1024;

struct SelectState {
    unsigned long long rank;                 // wanted rank among the entries that match `prefix`
    unsigned long long count;                // number of entries that match `prefix`
    uint32_t prefix;                         // the key bits fixed so far (lower bits zero)
    uint32_t fixed_bits;                     // how many top bits of the key are fixed
    uint32_t ncand;                          // candidates collected
    uint32_t tau_key;
    unsigned long long pad[4];
};
static_assert(sizeof(SelectState) == 64, "state is one 64-byte block");

struct Workspace {
    SelectState* st;
    unsigned long long* hist;                // [kBins]
    uint32_t* cand_key;                      // [kCap]
    unsigned long long* cand_idx;            // [kCap] linear index into the maps
};

__host__ __device__ inline Workspace carve(void* p)
{
    Workspace w;
    char* c = reinterpret_cast<char*>(p);
    w.st = reinterpret_cast<SelectState*>(c);
    w.hist = reinterpret_cast<unsigned long long*>(c + 64);
    w.cand_key = reinterpret_cast<uint32_t*>(c + 64 + (size_t)kBins * 8);
    w.cand_idx = reinterpret_cast<unsigned long long*>(c + 64 + (size_t)kBins * 8 + (size_t)kCap * 4);
    return w;
}
constexpr size_t kWorkspaceBytes = 64 + (size_t)kBins * 8 + (size_t)kCap * 4 + (size_t)kCap * 8;

__device__ __forceinline__ uint32_t key_of(float v)
{
    uint32_t b = __float_as_uint(v);
    if ((b << 1) == 0) b = 0;                                // -0 -> +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float value_of(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

__global__ void select_init_kernel(Workspace w, unsigned long long rank, unsigned long long n,
                                   float* tau_out, int none)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kBins; i += gridDim.x * blockDim.x) w.hist[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        w.st->rank = rank;
        w.st->count = n;
        w.st->prefix = 0;
        w.st->fixed_bits = 0;
        w.st->ncand = 0;
        w.st->tau_key = 0;
        if (none && tau_out) *tau_out = INFINITY;            // rank N: everything is pruned
    }
}

// The maps are walked in units, one wavefront per unit, all of (nearly) the same size so that
// any dealing of units to wavefronts is balanced: a unit is one row, or, for a causal map, the
// pair of rows i and Lq-1-i of a head, whose visible prefixes together hold Lk + (Lk - Lq) + 1
// entries whatever i is.  Inside a unit the two prefixes are laid end to end (the first padded
// to a multiple of 4 positions, so that no quad of positions spans both rows and 128-bit loads
// stay aligned) and lane l takes the 4 entries at position 256 * step + 4 * l.  All row
// arithmetic is wave-uniform.
struct Walk {
    const float* abar;
    long long units;
    int H, Lq, Lk;
    int causal;
    int per_head;                // units per head
};

struct Unit {                    // wave-uniform
    const float* row[2];
    long long base[2];           // linear index of the first entry of each row
    int n[2];                    // visible entries of each row (n[1] = 0: single row)
    int p0;                      // n[0] padded
    int total;                   // p0 + n[1]
};

__device__ __forceinline__ Unit decode_unit(const Walk& w, long long unit)
{
    Unit u;
    const int h = (int)(unit / w.per_head);
    const int t = (int)(unit - (long long)h * w.per_head);
    const long long off = (long long)w.Lk - w.Lq;
    const int i0 = t;
    const int i1 = w.causal ? w.Lq - 1 - t : t;
    u.n[0] = w.causal ? (int)min((long long)w.Lk, i0 + off + 1) : w.Lk;
    u.n[1] = (w.causal && i1 != i0) ? (int)min((long long)w.Lk, i1 + off + 1) : 0;
    u.base[0] = ((long long)h * w.Lq + i0) * w.Lk;
    u.base[1] = ((long long)h * w.Lq + i1) * w.Lk;
    u.row[0] = w.abar + u.base[0];
    u.row[1] = w.abar + u.base[1];
    u.p0 = (u.n[0] + 3) & ~3;                                // positions come in quads
    u.total = u.p0 + u.n[1];
    return u;
}

struct Quad {
    float4 v;
    int col;                     // column of the first entry
    int cnt;                     // how many of the 4 entries are visible entries of the row (0..4)
    int which;                   // 0 or 1: row of the unit
};

// U quads of this lane, starting at position pos0 of the unit.  The 128-bit loads of complete
// quads are issued back to back; quads cut by the end of a prefix are filled in afterwards.
template <int U>
__device__ __forceinline__ void load_quads(const Walk& w, const Unit& u, int pos0, int lane, Quad* q)
{
    const bool vec_ok = (w.Lk & 3) == 0;
    const float* p[U];
    bool full[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
        const int pos = pos0 + k * 256 + lane * 4;
        const bool second = pos >= u.p0;
        q[k].which = second ? 1 : 0;
        q[k].col = second ? pos - u.p0 : pos;
        const int nrow = second ? u.n[1] : u.n[0];
        int cnt = nrow - q[k].col;
        cnt = cnt < 0 ? 0 : (cnt > 4 ? 4 : cnt);
        q[k].cnt = cnt;
        p[k] = (second ? u.row[1] : u.row[0]) + q[k].col;
        full[k] = vec_ok && cnt == 4;
        q[k].v = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (vec_ok) {                                            // then the map holds at least 4 floats
#pragma unroll
        for (int k = 0; k < U; ++k) q[k].v = *reinterpret_cast<const float4*>(full[k] ? p[k] : w.abar);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
        if (full[k] || q[k].cnt == 0) continue;
        float e[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c < q[k].cnt) e[c] = p[k][c];
        q[k].v = make_float4(e[0], e[1], e[2], e[3]);
    }
}

template <int LEVEL> struct Digit;
template <> struct Digit<0> { static constexpr int shift = 17, bits = 15; };
template <> struct Digit<1> { static constexpr int shift = 2, bits = 15; };
template <> struct Digit<2> { static constexpr int shift = 0, bits = 2; };

template <int LEVEL>
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(Walk w, Workspace ws)
{
    constexpr int SHIFT = Digit<LEVEL>::shift, BITS = Digit<LEVEL>::bits;
    constexpr int NB = 1 << BITS;
    constexpr int U = 8;
    if (LEVEL > 0 && ws.st->count <= kCap) return;           // the candidates fit: no further digit needed
    __shared__ uint32_t h[NB];
    for (int i = threadIdx.x; i < NB; i += kThreads) h[i] = 0;
    __syncthreads();
    const uint32_t prefix = ws.st->prefix;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * (kThreads / 64);
    auto count = [&](float v) {
        const uint32_t key = key_of(v);
        bool match = true;
        if constexpr (LEVEL > 0) match = (key >> (SHIFT + BITS)) == (prefix >> (SHIFT + BITS));
        if (match) atomicAdd(&h[(key >> SHIFT) & (NB - 1)], 1u);
    };
    for (long long unit = (long long)wave * gridDim.x + blockIdx.x; unit < w.units; unit += nwaves) {
        const Unit u = decode_unit(w, unit);
        for (int pos0 = 0; pos0 < u.total; pos0 += 256 * U) {
            Quad q[U];
            load_quads<U>(w, u, pos0, lane, q);
#pragma unroll
            for (int k = 0; k < U; ++k) {
                if (q[k].cnt > 0) count(q[k].v.x);
                if (q[k].cnt > 1) count(q[k].v.y);
                if (q[k].cnt > 2) count(q[k].v.z);
                if (q[k].cnt > 3) count(q[k].v.w);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < NB; i += kThreads)
        if (h[i]) atomicAdd(&ws.hist[i], (unsigned long long)h[i]);
}


// One workgroup: find the bin whose cumulative count passes the wanted rank, fix that digit,
// and clear the histogram for the next level.  The histogram goes through LDS in two halves so
// that global memory is read and cleared with consecutive addresses per wavefront while every
// thread scans a run of consecutive bins.
template <int LEVEL>
__global__ __launch_bounds__(kThreads) void radix_select_kernel(Workspace ws)
{
    constexpr int SHIFT = Digit<LEVEL>::shift, BITS = Digit<LEVEL>::bits;
    constexpr int NB = 1 << BITS;
    constexpr int HALF = NB >= 2 * kThreads ? NB / 2 : NB;   // bins staged at a time
    constexpr int NHALF = NB / HALF;
    constexpr int PER = (HALF + kThreads - 1) / kThreads;    // consecutive bins per thread
    if (LEVEL > 0 && ws.st->count <= kCap) return;
    __shared__ unsigned long long bins[HALF];
    __shared__ unsigned long long part[kThreads];
    __shared__ unsigned long long group[32];
    __shared__ unsigned long long total;
    const int t = threadIdx.x;
    unsigned long long rank = ws.st->rank;
    const uint32_t prefix = ws.st->prefix;
    bool found = false;
    for (int half = 0; half < NHALF; ++half) {
        __syncthreads();                                     // LDS of the previous half is no longer read
        for (int i = t; i < HALF; i += kThreads) {
            bins[i] = ws.hist[half * HALF + i];
            ws.hist[half * HALF + i] = 0;
        }
        __syncthreads();
        if (found) continue;                                 // the remaining half is only cleared
        unsigned long long mine = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (t * PER + i < HALF) mine += bins[t * PER + i];
        part[t] = mine;
        __syncthreads();
        if (t < 32) {                                        // two-level exclusive scan of part[]
            unsigned long long s = 0;
            for (int i = 0; i < 32; ++i) s += part[t * 32 + i];
            group[t] = s;
        }
        __syncthreads();
        unsigned long long before = 0;
        for (int i = 0; i < (t >> 5); ++i) before += group[i];
        for (int i = (t & ~31); i < t; ++i) before += part[i];
        if (t == kThreads - 1) total = before + mine;
        if (rank >= before && rank < before + mine) {        // at most one thread, in one half
            unsigned long long cum = before;
            for (int i = 0; i < PER; ++i) {
                const unsigned long long c = bins[t * PER + i];
                if (rank < cum + c) {
                    ws.st->prefix = prefix | ((uint32_t)(half * HALF + t * PER + i) << SHIFT);
                    ws.st->fixed_bits = 32 - SHIFT;
                    ws.st->rank = rank - cum;
                    ws.st->count = c;
                    break;
                }
                cum += c;
            }
        }
        __syncthreads();
        if (rank < total) found = true;                      // uniform: every thread reads the same total
        else rank -= total;
    }
}

// Second sweep: the mask of every entry that the fixed key bits already decide, and the list of
// the entries they do not decide.  Candidates are staged per wavefront in LDS (a lane reserves
// room for its own with one LDS atomic) and moved to the global list in blocks, so the global
// counter sees one atomic per few hundred candidates.
constexpr int kStage = 384;                  // staged candidates per wavefront
constexpr int kStageFlush = kStage - 256;    // a quad step adds at most 64 lanes x 4 entries

__global__ __launch_bounds__(kThreads) void mask_collect_kernel(Walk w, Workspace ws, uint8_t* mask, int none)
{
    constexpr int U = 4;
    __shared__ uint32_t s_key[kThreads / 64][kStage];
    __shared__ unsigned long long s_idx[kThreads / 64][kStage];
    __shared__ uint32_t s_fill[kThreads / 64];
    const uint32_t fixed = ws.st->fixed_bits;
    const uint32_t prefix = ws.st->prefix;
    const bool exact = fixed == 32;                          // tau = prefix, nothing to collect
    const int shift = (exact || none) ? 0 : 32 - (int)fixed; // undecided low bits (2 .. 17)
    const uint32_t phi = prefix >> shift;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * (kThreads / 64);
    const bool vec_ok = (w.Lk & 3) == 0;
    if (lane == 0) s_fill[wave] = 0;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");

    auto flush = [&]() {                                     // wave-uniform
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");   // staged entries written by other lanes
        const int fill = (int)__builtin_amdgcn_readfirstlane(s_fill[wave]);
        if (fill == 0) return;
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&ws.st->ncand, (uint32_t)fill);
        base = __shfl(base, 0, 64);
        for (int i = lane; i < fill; i += 64) {
            const uint32_t slot = base + i;
            if (slot < kCap) {                               // always: the bin was chosen to fit
                ws.cand_key[slot] = s_key[wave][i];
                ws.cand_idx[slot] = s_idx[wave][i];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        if (lane == 0) s_fill[wave] = 0;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    };

    for (long long unit = (long long)wave * gridDim.x + blockIdx.x; unit < w.units; unit += nwaves) {
        const Unit u = decode_unit(w, unit);
        for (int pos0 = 0; pos0 < u.total && !none; pos0 += 256 * U) {
            Quad q[U];
            load_quads<U>(w, u, pos0, lane, q);
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const float ve[4] = {q[k].v.x, q[k].v.y, q[k].v.z, q[k].v.w};
                uint32_t out = 0;
                uint32_t keys[4];
                uint32_t cmask = 0;                          // which of the 4 entries are candidates
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool vis = e < q[k].cnt;
                    keys[e] = key_of(ve[e]);
                    const uint32_t hi = keys[e] >> shift;
                    if (vis && (exact ? keys[e] >= prefix : hi > phi)) out |= 1u << (8 * e);
                    if (vis && !exact && hi == phi) cmask |= 1u << e;
                }
                const long long lin = u.base[q[k].which] + q[k].col;
                if (__ballot(cmask != 0) != 0) {             // rare enough to keep out of the common path
                    if (__builtin_amdgcn_readfirstlane(s_fill[wave]) > kStageFlush) flush();
                    if (cmask != 0) {
                        uint32_t pos = atomicAdd(&s_fill[wave], (uint32_t)__popc(cmask));
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (cmask & (1u << e)) {
                                s_key[wave][pos] = keys[e];
                                s_idx[wave][pos] = (unsigned long long)(lin + e);
                                ++pos;
                            }
                    }
                }
                // candidates get 0 here, their byte comes later; a quad cut by the visible prefix
                // also writes the zeros of its hidden entries (inside the row)
                if (mask && q[k].cnt > 0) {
                    uint8_t* dst = mask + lin;
                    if (vec_ok) {
                        *reinterpret_cast<uint32_t*>(dst) = out;
                    } else {
                        for (int e = 0; e < q[k].cnt; ++e) dst[e] = (uint8_t)((out >> (8 * e)) & 1u);
                    }
                }
            }
        }
        // zeros for everything the sweep above did not write: the hidden tail of each row
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const bool present = r == 0 || u.base[1] != u.base[0];
            if (!present || !mask) continue;
            int start = none ? 0 : u.n[r];
            if (vec_ok) start = none ? 0 : (start + 3) & ~3;
            uint8_t* dst = mask + u.base[r];
            if (vec_ok) {
                for (int j = start + lane * 4; j < w.Lk; j += 256) *reinterpret_cast<uint32_t*>(dst + j) = 0u;
            } else {
                for (int j = start + lane; j < w.Lk; j += 64) dst[j] = 0;
            }
        }
    }
    flush();
}

// One workgroup: tau among the candidates, by radix selection over their undecided low bits.
__global__ __launch_bounds__(kThreads) void candidate_select_kernel(Workspace ws, float* tau_out)
{
    __shared__ uint32_t h[1024];
    __shared__ uint32_t group[32];
    __shared__ uint32_t chosen[2];                           // bin, count before it
    const int t = threadIdx.x;
    uint32_t prefix = ws.st->prefix;
    int remaining = 32 - (int)ws.st->fixed_bits;             // undecided low bits
    uint32_t rank = (uint32_t)ws.st->rank;                   // < ncand <= kCap
    const uint32_t n = min(ws.st->ncand, kCap);
    while (remaining > 0) {
        const int bits = remaining > 10 ? 10 : remaining;
        const int shift = remaining - bits;
        h[t] = 0;
        __syncthreads();
        for (uint32_t i0 = 0; i0 < n; i0 += 8 * kThreads) {   // 8 loads in flight per thread
            uint32_t keys[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t i = i0 + u * kThreads + t;
                keys[u] = ws.cand_key[i < n ? i : 0];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t i = i0 + u * kThreads + t;
                // remaining <= 17, so the shifts are defined
                if (i < n && (keys[u] >> remaining) == (prefix >> remaining))
                    atomicAdd(&h[(keys[u] >> shift) & ((1u << bits) - 1u)], 1u);
            }
        }
        __syncthreads();
        if (t < 32) {
            uint32_t s = 0;
            for (int i = 0; i < 32; ++i) s += h[t * 32 + i];
            group[t] = s;
        }
        __syncthreads();
        uint32_t before = 0;
        for (int i = 0; i < (t >> 5); ++i) before += group[i];
        for (int i = (t & ~31); i < t; ++i) before += h[i];
        const uint32_t mine = h[t];
        if (rank >= before && rank < before + mine) {        // exactly one thread
            chosen[0] = (uint32_t)t;
            chosen[1] = before;
        }
        __syncthreads();
        prefix |= chosen[0] << shift;
        rank -= chosen[1];
        remaining = shift;
        __syncthreads();
    }
    if (t == 0) {
        ws.st->tau_key = prefix;
        if (tau_out) *tau_out = value_of(prefix);
    }
}

__global__ __launch_bounds__(256) void candidate_fixup_kernel(Workspace ws, uint8_t* mask)
{
    const uint32_t n = min(ws.st->ncand, kCap);
    const uint32_t tau_key = ws.st->tau_key;
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u)
        if (ws.cand_key[i] >= tau_key) mask[ws.cand_idx[i]] = 1;
}

}  // namespace

size_t prune_mask_workspace_bytes() { return kWorkspaceBytes; }

hipError_t launch_prune_mask(const float* abar, int H, int Lq, int Lk, int causal,
                             unsigned long long rank, unsigned long long n, bool none, uint8_t* mask,
                             float* tau_out, void* workspace, hipStream_t stream)
{
    const Workspace ws = carve(workspace);
    Walk w;
    w.abar = abar;
    w.H = H;
    w.Lq = Lq;
    w.Lk = Lk;
    w.causal = causal;
    w.per_head = causal ? (Lq + 1) / 2 : Lq;
    w.units = (long long)H * w.per_head;
    const long long wg_units = (w.units + kThreads / 64 - 1) / (kThreads / 64);
    // the histogram takes 128 KB of LDS: one workgroup of 16 wavefronts per compute unit
    const unsigned grid = (unsigned)min((long long)256, wg_units);
    const unsigned grid2 = (unsigned)min((long long)512, wg_units);   // 48 KB of LDS: two per compute unit
    const int none_i = none ? 1 : 0;

    hipLaunchKernelGGL(select_init_kernel, dim3(32), dim3(256), 0, stream, ws, rank, n, tau_out, none_i);
    if (!none) {
        hipLaunchKernelGGL(radix_hist_kernel<0>, dim3(grid), dim3(kThreads), 0, stream, w, ws);
        hipLaunchKernelGGL(radix_select_kernel<0>, dim3(1), dim3(kThreads), 0, stream, ws);
        hipLaunchKernelGGL(radix_hist_kernel<1>, dim3(grid), dim3(kThreads), 0, stream, w, ws);
        hipLaunchKernelGGL(radix_select_kernel<1>, dim3(1), dim3(kThreads), 0, stream, ws);
        hipLaunchKernelGGL(radix_hist_kernel<2>, dim3(grid), dim3(kThreads), 0, stream, w, ws);
        hipLaunchKernelGGL(radix_select_kernel<2>, dim3(1), dim3(kThreads), 0, stream, ws);
    }
    hipLaunchKernelGGL(mask_collect_kernel, dim3(grid2), dim3(kThreads), 0, stream, w, ws, mask, none_i);
    if (!none) {
        hipLaunchKernelGGL(candidate_select_kernel, dim3(1), dim3(kThreads), 0, stream, ws, tau_out);
        if (mask) hipLaunchKernelGGL(candidate_fixup_kernel, dim3(256), dim3(256), 0, stream, ws, mask);
    }
    return hipGetLastError();
}

}  // namespace ap
