// Masked attention forward on the bf16 matrix cores (Section 3.2, masked-attention equation).
//
// One workgroup per block row of the layout (block_m = 32 * NW queries, one wavefront per 32
// queries).  The workgroup walks only the stored tiles of its block row.  Per tile:
//   1. the 64 key rows and 64 value rows go from HBM/L2 straight into LDS with 128-bit
//      buffer loads that write LDS directly (no staging registers); the loads of the next tile
//      (two LDS stages), or of the next tile's keys and this tile's values (one stage: half the
//      LDS, more workgroups per compute unit), are in flight while the current tile is computed;
//      LDS rows are unpadded and XOR-swizzled in 16-byte chunks so that both the key-operand
//      reads and the transposing value reads are bank-conflict free;
//   2. S^T = K Q^T on v_mfma_f32_32x32x16_bf16, so that every lane holds scores of ONE query
//      (lane % 32) for 32 of the 64 keys -- the row maximum is an in-register reduction plus
//      a single exchange with lane ^ 32, and the row sum needs no exchange until the end;
//   3. the lane's 64-bit bitmap word (and the causal limit) turns pruned scores into -inf in
//      registers, before the exponential; tiles whose visible part is all ones skip this;
//   4. online softmax in fp32 (exp2 with scale*log2(e) folded into one fma);
//   5. O^T += V^T P^T on the matrix cores: the S^T accumulator registers already have the
//      lane layout of the P^T operand, and V^T is read from the row-major LDS tile with the
//      transposing LDS read, so nothing is shuffled.
// O is normalised, staged through LDS and written with coalesced 128-bit stores, together with
// the optional log-sum-exp.
//
// Matrix-core register layouts used below (32x32x16, 64 lanes, l = lane):
//   A[m][k]: m = l % 32, k = 8*(l/32) + e, e = 0..7        B[k][n]: n = l % 32, same k
//   C[m][n]: n = l % 32, m = 8*(i/4) + 4*(l/32) + i%4, i = 0..15
// The contraction index of the second product runs over keys in the order the S^T registers
// hold them (slot (l/32, e) of 16-key step ks is key 16*ks + 8*(e/4) + 4*(l/32) + e%4); both
// operands use the same order, which leaves the sum unchanged.
//
// The transposing LDS read (ds_read_b64_tr_b16) works on groups of 16 lanes: lane i of a group
// supplies the address of 4 consecutive 16-bit elements, and receives element (i % 4) of the
// data addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With lanes 4j..4j+3 pointing at 16
// consecutive columns of row j, lane i ends up with column i of rows 0..3.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"
#include "ap_mfma_common.h"

namespace ap {

namespace {

using namespace mfma;

// SCHED = false: walk the stored tiles of the layout (64 consecutive keys each, causal limit
// applied here).  SCHED = true: walk the entries of a visit schedule (consecutive or gathered
// keys, causal limit already folded into the bitmaps).
// SPLIT = true: the entries of a block row are cut into a.splits contiguous chunks, one workgroup
// each, which write a normalised fp32 partial output and its log-sum-exp for merge_splits_kernel
// (few queries against many keys: one workgroup per block row would leave the chip idle).
//
// The leading scalar arguments repeat fields of `a` (row pointers, entry counts, block rows per head
// of the layout, heads, splits): the library is built with kernel-argument preloading, which hands
// the first 16 dwords of the argument block to a wavefront in registers when it starts, so the
// loads of the block row's pointer and count go out at once instead of after a first round trip
// for the argument block (the structure itself is too large to be preloaded).
template <int D, int NW, int STAGES, bool SCHED, bool SPLIT = false>
__global__ __launch_bounds__(64 * NW, (D <= 64 && STAGES == 1) ? 3 : 2) void fwd_mfma_kernel(
    const int32_t* __restrict__ p_row_ptr, const int32_t* __restrict__ p_cnt, int nQB, int xcd_chunk,
    int p_nqb_layout, int p_H, int p_splits, FwdArgs a)
{
    constexpr int BM = 32 * NW;
    constexpr int KSTEPS = D / 16;                           // contraction steps of Q K^T
    constexpr int DBLK = D / 32;                             // 32-wide blocks of the head dim
    constexpr int CPR = D / 8;                               // 16-byte chunks per row
    constexpr int TILE = kBN * D;                            // elements of one K or V tile
    constexpr int OSTAGE = BM * D;                           // elements needed to stage O
    constexpr int TILES = (STAGES * 2 * TILE > OSTAGE) ? STAGES * 2 * TILE : OSTAGE;
    // per-entry metadata travels through LDS like the tiles: two slots of bitmap words (BM x 8
    // bytes) and two slots of gather keys (64 x 4 bytes)
    constexpr int META_W = BM * 4;                           // elements (2 bytes) of one word slot
    constexpr int META_C = 128;                              // elements of one key slot
    constexpr int SMEM = TILES + 2 * META_W + 2 * META_C;

    __shared__ __attribute__((aligned(1024))) uint16_t smem[SMEM];
    lds_u16* lds = (lds_u16*)smem;
    lds_u16* wmeta = lds + TILES;
    lds_u16* cmeta = wmeta + 2 * META_W;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
    const int lane = tid & 63;
    const int n = lane & 31;                                 // query inside the wavefront's 32
    const int hh = lane >> 5;                                // which half of the key slots

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // (batch, head) pairs so that the block rows sharing K and V also share an L2.
    int bid = blockIdx.x;
    if (xcd_chunk > 0) bid = (bid & 7) * xcd_chunk + (bid >> 3);
    int split = 0;
    if (SPLIT) {
        split = bid % p_splits;
        bid /= p_splits;
    }
    const int qb = nQB - 1 - (bid % nQB);                    // long causal rows first
    const int h = (bid / nQB) % p_H;
    const int b = bid / (nQB * p_H);
    const int r = h * p_nqb_layout + qb;                     // requested first: everything else waits for these
    int t_begin = p_row_ptr[r];
    int nt = SCHED ? p_cnt[r] : p_row_ptr[r + 1] - t_begin;

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* Op = (uint16_t*)a.O + (size_t)b * a.so[0] + (size_t)h * a.so[1];
    const int sk_bytes = (int)a.sk[2] * 2, sv_bytes = (int)a.sv[2] * 2;
    // rows >= Lk lie beyond num_records: the hardware returns zeros for them
    const rsrc_t k_rsrc = make_rsrc(Kp, (unsigned)((a.Lk - 1) * sk_bytes + D * 2));
    const rsrc_t v_rsrc = make_rsrc(Vp, (unsigned)((a.Lk - 1) * sv_bytes + D * 2));

    const int brow = wave * 32 + n;                          // row inside the block row
    const int qrow = qb * BM + brow;                         // this lane's query
    const bool row_ok = qrow < a.Lq;

    // Q^T operand, resident in registers for the whole kernel
    bf16x8 qreg[KSTEPS];
    {
        const uint16_t* qr = Qp + (size_t)(row_ok ? qrow : a.Lq - 1) * a.sq[2] + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            qreg[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
    }

    f32x16 oacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m = -INFINITY;                                     // running max of raw scores
    float lsum = 0.f;                                        // this lane's share of the row sum
    const float sc = a.scale * kLog2e;

    if (SPLIT) {                                             // this workgroup's chunk of the entries
        const int chunk = (nt + a.splits - 1) / a.splits;
        const int e0 = min(nt, split * chunk);
        t_begin += e0;
        nt = min(nt - e0, chunk);
    }
    const long long off = (long long)a.Lk - a.Lq;
    const long long diag = (long long)qrow + off;            // last visible key if causal
    const uint64_t* words = SCHED ? a.sched.bitmaps : a.bitmaps;
    constexpr int NLOAD = (D / 8) / NW;                      // load instructions per wavefront and operand
    constexpr int RPI = 64 / (D / 8);                        // tile rows per load instruction
    const int g_row = lane / (D / 8);                        // this lane's row inside a load instruction

    // The first key of every tile of the block row (>= 0, or -1 for a gathered entry) is kept in
    // registers, one tile per lane and 128 tiles at a time, and handed out with v_readlane: a
    // memory load of a start inside the loop would have to be waited for, and that wait would
    // also cover the tile loads issued just before it.
    const int32_t* starts_mem = SCHED ? a.sched.start : a.col_idx;
    const int nt_stored = nt;
    auto load_starts = [&](int base) -> int {
        int v = 0x7fffffff;
        if (base + lane < nt_stored) {
            v = starts_mem[t_begin + base + lane];
            if (!SCHED) v *= kBN;
        }
        return v;
    };
    int starts_lo = load_starts(0), starts_hi = load_starts(64);
    int starts_base = 0;                                     // tile held by lane 0 of starts_lo
    if (!SCHED && a.causal) {                                // drop tiles that are entirely in the future
        const long long block_diag = (long long)qb * BM + (BM - 1) + off;
        int visible = 0;                                     // columns ascend: the visible tiles come first
        for (int base = 0; base < nt_stored; base += 64) {
            const int v = base == 0 ? starts_lo : (base == 64 ? starts_hi : load_starts(base));
            visible += __popcll(__ballot((long long)v <= block_diag));
        }
        nt = visible;
    }
    auto tile_start = [&](int i) -> int {                    // i is uniform, starts_base <= i
        if (i - starts_base >= 128) {                        // once per 64 tiles beyond the first 128
            starts_lo = starts_hi;
            starts_base += 64;
            starts_hi = load_starts(starts_base + 64);
            asm volatile("" : "+v"(starts_hi));              // take the load's wait here, not in every iteration
        }
        const int rel = i - starts_base;
        return rel < 64 ? __builtin_amdgcn_readlane(starts_lo, rel)
                        : __builtin_amdgcn_readlane(starts_hi, rel - 64);
    };
    // Metadata of entry i of this block row, moved to LDS by wavefront 0 with the same kind of
    // load as the tiles (so the loop holds no load that returns to registers, whose wait would
    // also cover the tile loads in flight): its bitmap words, and its 64 gather keys.
    const rsrc_t w_rsrc = make_rsrc(words + (size_t)t_begin * BM, (unsigned)nt_stored * BM * 8u);
    const rsrc_t c_rsrc = make_rsrc(SCHED ? a.sched.cols + (size_t)t_begin * 64 : nullptr,
                                    SCHED ? (unsigned)nt_stored * 256u : 0u);
    auto dma_words = [&](int i, int slot) {
        if (wave == 0 && lane < BM / 2)
            load16_to_lds(lds_addr_of(wmeta + slot * META_W), lane * 16, w_rsrc, i * BM * 8);
    };
    auto dma_cols = [&](int i, int slot) {
        if (wave == 0 && lane < 16)
            load16_to_lds(lds_addr_of(cmeta + slot * META_C), lane * 16, c_rsrc, i * 256);
    };
    auto read_word = [&](int slot) -> uint64_t {
        return *reinterpret_cast<const uint64_t*>(smem + TILES + slot * META_W + brow * 4);
    };
    // keys of the rows this lane loads, for a gathered entry
    auto read_cols = [&](int slot, int* gk) {
#pragma unroll
        for (int u = 0; u < NLOAD; ++u)
            gk[u] = *reinterpret_cast<const int*>(smem + TILES + 2 * META_W + slot * META_C +
                                                  ((wave + NW * u) * RPI + g_row) * 2);
    };
    auto issue_tile = [&](int start, const int* gidx, lds_u16* Kd) {
        if (!SCHED || start >= 0) {
            issue_tile_loads<D, NW, false>(k_rsrc, Kd, start, sk_bytes, wave, lane);
            issue_tile_loads<D, NW, true>(v_rsrc, Kd + TILE, start, sv_bytes, wave, lane);
        } else {
            issue_gather_loads<D, NW, false>(k_rsrc, Kd, gidx, sk_bytes, wave, lane);
            issue_gather_loads<D, NW, true>(v_rsrc, Kd + TILE, gidx, sv_bytes, wave, lane);
        }
    };

    // per-lane LDS read offsets (elements), loop invariant
    const int k_swz = (hh ^ swz_k<D>(n));                    // rows n and n + 32 share the swizzle
    const int i16 = lane & 15, g = (lane >> 4) & 1, vj = i16 >> 2;
    const int v_lane_row = 4 * hh + vj;
    const int v_in_chunk = 4 * (i16 & 1);
    const int v_chunk_lo = 2 * g + ((i16 >> 1) & 1);
    const int v_swz = swz_v<D>(vj) >> 2;                     // xor on the 4-chunk group index

    // ---- the three pieces of work on one tile, shared by both pipelines below

    // S^T = K Q^T : two 32-key blocks.  Key operands are requested from LDS two groups ahead of
    // the matrix instructions that consume them (a group = 2 contraction steps x 2 key blocks),
    // so LDS latency is paid once per tile while only three groups are live in registers.
    auto qk_tile = [&](lds_u16* Ks, f32x16* sacc) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
        constexpr int GS = (KSTEPS >= 4) ? 2 : 1;            // contraction steps per group
        constexpr int NG = KSTEPS / GS;                      // groups
        bf16x8 kreg[KSTEPS][2];
        auto read_group = [&](int gi) {
#pragma unroll
            for (int kk = gi * GS; kk < (gi + 1) * GS; ++kk)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    kreg[kk][kb] = *reinterpret_cast<const bf16x8*>(
                        (const uint16_t*)Ks + (kb * 32 + n) * D + ((2 * kk) ^ k_swz) * 8);
        };
        auto mfma_group = [&](int gi) {
#pragma unroll
            for (int kk = gi * GS; kk < (gi + 1) * GS; ++kk)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[kk][kb], qreg[kk], sacc[kb], 0, 0, 0);
        };
        read_group(0);
        if (NG > 1) read_group(1);
        // matrix instructions of this wavefront go ahead of the vector work of the others on the SIMD
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            if (gi + 2 < NG) read_group(gi + 2);
            mfma_group(gi);
        }
        __builtin_amdgcn_s_setprio(0);
        // pin that order: reads of two groups, then (reads of the next group, matrix ops of this one)
        __builtin_amdgcn_sched_group_barrier(0x100, (NG > 1 ? 2 : 1) * 2 * GS, 0);
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            if (gi + 2 < NG) __builtin_amdgcn_sched_group_barrier(0x100, 2 * GS, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2 * GS, 0);
        }
    };

    // Mask in registers, row maximum, online softmax; leaves P in sacc.
    auto softmax_tile = [&](uint64_t word, f32x16* sacc) {
        float tmax = -INFINITY;
        if (__ballot(word != ~0ull) == 0) {                  // every visible entry kept: no selects
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sacc[kb][i]);
        } else {
            const uint64_t wsh = word >> (4 * hh);
            const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int pos = 8 * (i / 4) + (i % 4);
                    // all-ones where kept (signed one-bit field), then a bit-select between the
                    // score and -inf: two vector instructions and no condition code
                    const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)wbits[kb], pos, 1);
                    const float sv = __uint_as_float((__float_as_uint(sacc[kb][i]) & keep) | (0xff800000u & ~keep));
                    sacc[kb][i] = sv;
                    tmax = fmaxf(tmax, sv);
                }
        }
        {   // the other half of this query's keys lives in lane ^ 32: one swap of the wave halves
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
            tmax = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
        }

        // Online softmax with a lazily updated reference.  m is the reference the exponentials
        // are taken against; it only moves up when this tile's row maximum exceeds it by more
        // than kLazy in the log2 domain, so P stays below 2^kLazy (harmless in bf16/fp32) and the
        // rescaling of O, 16*D/32 multiplies per lane, becomes rare.  The result is the same
        // quotient sum(p v) / sum(p) whatever reference is used.
        const bool grow = (tmax - m) * sc > kLazy;           // m = -inf: any finite tmax grows it
        if (__ballot(grow) != 0) {
            // rows that keep their reference get exactly 1 (also when it still is -inf)
            const float alpha = grow ? __builtin_amdgcn_exp2f((m - tmax) * sc) : 1.0f;   // 0 from -inf
            m = grow ? tmax : m;
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        }
        const float msc = (m == -INFINITY) ? 0.f : m * sc;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], sc, -msc));
                sacc[kb][i] = pe;
                psum += pe;
            }
        lsum += psum;
    };

    // O^T += V^T P^T : the value operands of 16-key step ks + 1 are requested from LDS before the
    // matrix instructions of step ks are issued.
    auto pv_tile = [&](lds_u16* Vs, const f32x16* sacc) {
        auto read_v = [&](int ks, bf16x8* vreg) {
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                const int chunk = ((db ^ v_swz) << 2) + v_chunk_lo;
                lds_u16* p0 = Vs + (16 * ks + v_lane_row) * D + chunk * 8 + v_in_chunk;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p0);
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 8 * D));
                vreg[db] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        bf16x8 vcur[DBLK], vnext[DBLK];
        read_v(0, vcur);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 pb;
#pragma unroll
            for (int e = 0; e < 8; ++e) pb[e] = (__bf16)sacc[ks >> 1][8 * (ks & 1) + e];
            if (ks + 1 < 4) read_v(ks + 1, vnext);
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vcur[db], pb, oacc[db], 0, 0, 0);
#pragma unroll
            for (int db = 0; db < DBLK; ++db) vcur[db] = vnext[db];
        }
        __builtin_amdgcn_s_setprio(0);
    };

    auto apply_causal = [&](uint64_t word, int k0) -> uint64_t {
        if (!SCHED && a.causal) {
            const long long lim = diag - k0;
            if (lim < 0) word = 0;
            else if (lim < 63) word &= (2ull << lim) - 1ull;
        }
        return word;
    };
    // A layout built for more keys than this call has (a fixed mask, a shorter sequence): the slots
    // of an entry whose key exists.  slot = the metadata slot that holds the entry's gather keys;
    // must be called before that slot is handed to a later entry.
    auto crop_valid = [&](int k0, int slot) -> uint64_t {
        if (!a.crop) return ~0ull;                           // uniform
        if (!SCHED || k0 >= 0) {
            const long long lim = (long long)a.Lk - 1 - k0;
            return lim < 0 ? 0ull : (lim < 63 ? (2ull << lim) - 1ull : ~0ull);
        }
        const int key = *reinterpret_cast<const int*>(smem + TILES + 2 * META_W + slot * META_C + lane * 2);
        return __ballot(key < a.Lk);
    };

    int gidx[NLOAD];                                         // gather keys of the next tile to be issued
#pragma unroll
    for (int u = 0; u < NLOAD; ++u) gidx[u] = 0;
    // First use of the Q registers, placed before the loops: the wait that the compiler attaches
    // to the first use of a loaded register would otherwise sit inside the loop, in front of the
    // first matrix instruction, and there it would also wait for the tile loads just issued.
    auto settle_q = [&]() {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) asm volatile("" : "+v"(qreg[kk]));
    };

    if constexpr (STAGES == 2) {
        // ---- Pipeline A: two LDS stages of (K, V); the whole next tile is in flight while the
        // current one is computed; one barrier per tile.
        int k0_next = 0;                                     // start of the tile whose loads were issued last
        if (nt > 0) {
            k0_next = tile_start(0);
            if (SCHED && k0_next < 0) {                      // the very first entry is gathered: fetch its keys
                dma_cols(0, 0);
                wait_vmem();
                __syncthreads();
                read_cols(0, gidx);
            }
            issue_tile(k0_next, gidx, lds);
            dma_words(0, 0);
            if (SCHED && nt > 1 && tile_start(1) < 0) dma_cols(1, 1);
        }
        settle_q();
        for (int it = 0; it < nt; ++it) {
            const int stage = it & 1;
            lds_u16* Ks = lds + stage * 2 * TILE;
            lds_u16* Vs = Ks + TILE;
            const int k0 = k0_next;

            wait_vmem();                                     // my loads of this tile have landed
            __syncthreads();                                 // ... and everybody else's
            uint64_t word = read_word(stage) & crop_valid(k0, stage);
            if (it + 1 < nt) {
                k0_next = tile_start(it + 1);
                if (SCHED && k0_next < 0) read_cols(stage ^ 1, gidx);
                issue_tile(k0_next, gidx, lds + (stage ^ 1) * 2 * TILE);
                dma_words(it + 1, stage ^ 1);
                if (SCHED && it + 2 < nt && tile_start(it + 2) < 0) dma_cols(it + 2, stage);
            }
            word = apply_causal(word, k0);
            if (__ballot(word != 0) != 0) {                  // something visible for these 32 queries
                f32x16 sacc[2];
                qk_tile(Ks, sacc);
                softmax_tile(word, sacc);
                pv_tile(Vs, sacc);
            }
        }
    } else {
        // ---- Pipeline B: one K buffer and one V buffer (half the LDS, twice the workgroups per
        // CU).  V of the current tile is requested as soon as every wavefront is past the previous
        // tile's second product and travels under Q K^T and the softmax; K of the next tile is
        // requested as soon as every wavefront has its scores and travels under the softmax and
        // the second product.  Three barriers per tile.
        lds_u16* Ks = lds;
        lds_u16* Vs = lds + TILE;
        int gcur[NLOAD];                                     // gather keys of the current tile (for its V)
#pragma unroll
        for (int u = 0; u < NLOAD; ++u) gcur[u] = 0;
        int s_cur = 0, s_nxt = 0;                            // starts of tile it and tile it + 1
        if (nt > 0) {
            s_cur = tile_start(0);
            if (SCHED && s_cur < 0) {                        // the very first entry is gathered: fetch its keys
                dma_cols(0, 0);
                wait_vmem();
                __syncthreads();
                read_cols(0, gcur);
            }
            if (!SCHED || s_cur >= 0) issue_tile_loads<D, NW, false>(k_rsrc, Ks, s_cur, sk_bytes, wave, lane);
            else issue_gather_loads<D, NW, false>(k_rsrc, Ks, gcur, sk_bytes, wave, lane);
            dma_words(0, 0);
            if (nt > 1) {
                s_nxt = tile_start(1);
                if (SCHED && s_nxt < 0) dma_cols(1, 1);
            }
        }
        settle_q();
        for (int it = 0; it < nt; ++it) {
            const int slot = it & 1;
            wait_vmem();                                     // K and metadata of this tile (keys of the next)
            __syncthreads();                                 // ... for everybody; the V buffer is free
            const uint64_t valid = crop_valid(s_cur, slot);
            // metadata of later tiles first, so that only the K loads are younger than the V loads
            int s_nn = 0;
            if (it + 1 < nt) dma_words(it + 1, slot ^ 1);
            if (it + 2 < nt) {
                s_nn = tile_start(it + 2);
                if (SCHED && s_nn < 0) dma_cols(it + 2, slot);
            }
            if (!SCHED || s_cur >= 0) issue_tile_loads<D, NW, true>(v_rsrc, Vs, s_cur, sv_bytes, wave, lane);
            else issue_gather_loads<D, NW, true>(v_rsrc, Vs, gcur, sv_bytes, wave, lane);
            const uint64_t word = apply_causal(read_word(slot), s_cur) & valid;
            const bool active = __ballot(word != 0) != 0;    // something visible for these 32 queries
            f32x16 sacc[2];
            if (active) qk_tile(Ks, sacc);
            if (SCHED && it + 1 < nt && s_nxt < 0) read_cols(slot ^ 1, gidx);
            __syncthreads();                                 // the K buffer is free
            if (it + 1 < nt) {
                if (!SCHED || s_nxt >= 0) issue_tile_loads<D, NW, false>(k_rsrc, Ks, s_nxt, sk_bytes, wave, lane);
                else issue_gather_loads<D, NW, false>(k_rsrc, Ks, gidx, sk_bytes, wave, lane);
            }
            if (active) softmax_tile(word, sacc);
            // V of this tile has landed once at most the K loads just issued are outstanding
            if (it + 1 < nt) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NLOAD) : "memory");
            else wait_vmem();
            __syncthreads();
            if (active) pv_tile(Vs, sacc);
            s_cur = s_nxt;
            s_nxt = s_nn;
#pragma unroll
            for (int u = 0; u < NLOAD; ++u) gcur[u] = gidx[u];
        }
    }

    // ---- epilogue: normalise, stage O through LDS, coalesced stores; lse
    float ltot;                                              // both halves of the row sum
    {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lsum), __float_as_uint(lsum), false, false);
        ltot = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    if (SPLIT) {                                             // partial result: fp32, normalised by its own sum
        const size_t prow = (((size_t)split * a.B + b) * a.H + h) * a.Lq + qrow;
        if (row_ok) {
            float* po = a.part_o + prow * D;
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
                    *reinterpret_cast<float4*>(po + 32 * db + 8 * g4 + 4 * hh) =
                        make_float4(oacc[db][4 * g4] * inv, oacc[db][4 * g4 + 1] * inv,
                                    oacc[db][4 * g4 + 2] * inv, oacc[db][4 * g4 + 3] * inv);
            if (hh == 0)
                a.part_lse[prow] = ltot > 0.f ? (m * sc + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
        }
        return;
    }
    __syncthreads();                                         // all wavefronts are done with K/V in LDS
    uint16_t* ostage = smem + wave * 32 * D;                 // this wavefront's 32 rows
    {
        const int f = swz_k<D>(n);
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                uint2 w;
                w.x = pack_bf16_rne(oacc[db][4 * g4] * inv, oacc[db][4 * g4 + 1] * inv);
                w.y = pack_bf16_rne(oacc[db][4 * g4 + 2] * inv, oacc[db][4 * g4 + 3] * inv);
                const int chunk = (4 * db + g4) ^ f;
                *reinterpret_cast<uint2*>(ostage + n * D + chunk * 8 + 4 * hh) = w;
            }
    }
    // same wavefront reads back what it wrote: no barrier needed, only LDS ordering
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    {
        const int row_base = qb * BM + wave * 32;
#pragma unroll
        for (int u = 0; u < (32 * CPR) / 64; ++u) {
            const int idx = u * 64 + lane;
            const int rr = idx / CPR, c = idx % CPR;
            const uint4 v = *reinterpret_cast<const uint4*>(ostage + rr * D + (c ^ swz_k<D>(rr)) * 8);
            if (row_base + rr < a.Lq)
                *reinterpret_cast<uint4*>(Op + (size_t)(row_base + rr) * a.so[2] + c * 8) = v;
        }
    }
    if (a.lse && hh == 0 && row_ok)
        a.lse[((size_t)b * a.H + h) * a.Lq + qrow] =
            ltot > 0.f ? (m * sc + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
}

template <int D, int NW, int STAGES>
hipError_t launch_one(const FwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + 32 * NW - 1) / (32 * NW);
    const long long blocks = (long long)nQB * a.H * a.B;
    const int xcd_chunk = (blocks % 8 == 0) ? (int)(blocks / 8) : 0;
    const int32_t* cnt = a.sched.cnt;
    if (cnt)
        hipLaunchKernelGGL((fwd_mfma_kernel<D, NW, STAGES, true>), dim3((unsigned)blocks), dim3(64 * NW), 0,
                           stream, a.row_ptr, cnt, nQB, xcd_chunk, a.nqb_layout, a.H, a.splits, a);
    else
        hipLaunchKernelGGL((fwd_mfma_kernel<D, NW, STAGES, false>), dim3((unsigned)blocks), dim3(64 * NW), 0,
                           stream, a.row_ptr, cnt, nQB, xcd_chunk, a.nqb_layout, a.H, a.splits, a);
    return hipGetLastError();
}

// O = sum_s exp(lse_s - lse) O_s with lse = ln sum_s exp(lse_s): one thread per (row, 4 elements).
template <int D>
__global__ __launch_bounds__(256) void merge_splits_kernel(FwdArgs a)
{
    constexpr int TPR = D / 4;                               // threads per row
    const long long rows = (long long)a.B * a.H * a.Lq;
    const long long row = ((long long)blockIdx.x * 256 + threadIdx.x) / TPR;
    const int part = threadIdx.x % TPR;
    if (row >= rows) return;
    float mx = -INFINITY;
    for (int s = 0; s < a.splits; ++s) mx = fmaxf(mx, a.part_lse[(size_t)s * rows + row]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float tot = 0.f;
    if (mx != -INFINITY) {
        for (int s = 0; s < a.splits; ++s) {
            const float w = __expf(a.part_lse[(size_t)s * rows + row] - mx);   // 0 for an empty chunk
            if (w == 0.f) continue;                          // its partial output may be anything finite
            const float4 o = *reinterpret_cast<const float4*>(a.part_o + ((size_t)s * rows + row) * D + part * 4);
            acc.x = fmaf(w, o.x, acc.x);
            acc.y = fmaf(w, o.y, acc.y);
            acc.z = fmaf(w, o.z, acc.z);
            acc.w = fmaf(w, o.w, acc.w);
            tot += w;
        }
        const float inv = 1.f / tot;
        acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    }
    const int i = (int)(row % a.Lq);
    const long long bh = row / a.Lq;
    const int h = (int)(bh % a.H);
    const long long b = bh / a.H;
    uint16_t* dst = (uint16_t*)a.O + (size_t)b * a.so[0] + (size_t)h * a.so[1] + (size_t)i * a.so[2] + part * 4;
    uint2 w2;
    w2.x = pack_bf16_rne(acc.x, acc.y);
    w2.y = pack_bf16_rne(acc.z, acc.w);
    *reinterpret_cast<uint2*>(dst) = w2;
    if (a.lse && part == 0) a.lse[row] = mx == -INFINITY ? -INFINITY : mx + __logf(tot);
}

template <int D>
hipError_t launch_split_d(const FwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + 63) / 64;
    const long long blocks = (long long)nQB * a.H * a.B * a.splits;
    constexpr int ST = D == 128 ? 1 : 2;
    const int32_t* cnt = a.sched.cnt;
    if (cnt)
        hipLaunchKernelGGL((fwd_mfma_kernel<D, 2, ST, true, true>), dim3((unsigned)blocks), dim3(128), 0,
                           stream, a.row_ptr, cnt, nQB, 0, a.nqb_layout, a.H, a.splits, a);
    else
        hipLaunchKernelGGL((fwd_mfma_kernel<D, 2, ST, false, true>), dim3((unsigned)blocks), dim3(128), 0,
                           stream, a.row_ptr, cnt, nQB, 0, a.nqb_layout, a.H, a.splits, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long threads = (long long)a.B * a.H * a.Lq * (D / 4);
    hipLaunchKernelGGL(merge_splits_kernel<D>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_merge_splits(const FwdArgs& a, hipStream_t stream)
{
    const long long rows = (long long)a.B * a.H * a.Lq;
    switch (a.D) {
    case 32: hipLaunchKernelGGL(merge_splits_kernel<32>, dim3((unsigned)((rows * 8 + 255) / 256)), dim3(256), 0, stream, a); break;
    case 64: hipLaunchKernelGGL(merge_splits_kernel<64>, dim3((unsigned)((rows * 16 + 255) / 256)), dim3(256), 0, stream, a); break;
    case 128: hipLaunchKernelGGL(merge_splits_kernel<128>, dim3((unsigned)((rows * 32 + 255) / 256)), dim3(256), 0, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fwd_split(const FwdArgs& a, hipStream_t stream)
{
    switch (a.D) {
    case 32: return launch_split_d<32>(a, stream);
    case 64: return launch_split_d<64>(a, stream);
    case 128: return launch_split_d<128>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fwd_mfma(const FwdArgs& a, hipStream_t stream)
{
    // 64-query block rows: two wavefronts and one LDS stage at D = 128 (32 KB, four workgroups per
    // CU) and at D = 64 (16 KB and at most 168 registers: six workgroups per CU, which matters for
    // short sequences where a workgroup's life is mostly waiting for its first loads); two stages
    // at D = 32.
    // 128-query block rows: four wavefronts and two LDS stages, two workgroups per CU.
    const bool wide = a.block_m == 128;
    switch (a.D) {
    case 32: return wide ? launch_one<32, 4, 2>(a, stream) : launch_one<32, 2, 2>(a, stream);
    case 64: return wide ? launch_one<64, 4, 2>(a, stream) : launch_one<64, 2, 1>(a, stream);
    case 128: return wide ? launch_one<128, 4, 2>(a, stream) : launch_one<128, 2, 1>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ap
