// bf16 matrix-core forward kernel for sliding-window self-attention with a bounded window (Eq. (sliding
// window)), gfx950: one workgroup walks one (sequence, head) from its first key tile to its last.
//
// A query block (32 queries) needs the key tiles (32 keys) first(j) .. last(j) of its window, and consecutive
// blocks need consecutive, overlapping ranges: tile t is wanted by the blocks t - c_r .. t + c_l
// (c_l = ceil(left / 32), c_r = floor((31 + right) / 32)).  So the key tiles of the sequence stream ONCE through
// a ring of LDS stages, and at every step the c_l + c_r + 1 blocks whose windows cover the tile in flight work
// on it, each in a wave of its own.  When a block's last tile has passed, its wave writes the block's output
// rows during the next step and then takes the next unassigned block (block j runs in compute wave j mod NWC,
// NWC >= c_l + c_r + 2).  Against one workgroup per 128-query tile this removes the steps in which a wave only
// waits for the other waves' windows, lets output and query staging overlap with the other waves' arithmetic,
// and fetches every key / value row exactly once per (sequence, head).  It is the outer-loop pipelining of
// App. "GDPA and Fused PFFN Kernel" (work of consecutive outer iterations overlapped because the inner loops
// are short), arranged for 64-wide waves that share one compute unit's LDS.
//
// Wave 0 is the loader (it computes nothing): it sends key / value tiles ahead into a ring of LDS stages by
// buffer-load-to-LDS (lds_ring.h), counts its own loads (they complete in issue order) and publishes the number
// of tiles that have landed in an LDS word.  The waves of the workgroup do NOT meet at barriers in the key loop:
// a barrier per step would put every wave into the same phase at the same time (all on the matrix cores, then
// all on the vector ALU: measured 3.0 ms at the bench size, 2.3 ms with two shifted groups of waves), whereas
// waves that drift apart by a tile or two overlap the matrix-core phase of one with the vector phase of
// another on their SIMD.  Instead a compute wave waits (bounded polling of the LDS word) until its tile has
// landed, and publishes its own progress - the first tile it may still read - in a word of its own; the loader
// reuses a stage once every compute wave is past the tile it held.  A compute wave fetches the query fragments
// of its next block straight into registers during the last tile of the current one and transposes its output
// rows through a small LDS slot of its own, so nearly the whole LDS is ring: seven stages, three tiles in
// flight, the waves free to spread over the rest.
//
// Per tile and compute wave the arithmetic is that of the other forward kernels (S^T = K Q^T, online softmax
// in registers, O^T += V^T P^T through transposing LDS reads).
#include <type_traits>

#include "attn_fwd_score.h"
#include "lds_ring.h"

namespace kunlun {

template <int D, int NWC>
struct BandSmem {
    static constexpr int ROW = D * 2;
    static constexpr int TILE = KT * ROW;           // 32 rows of K or of V
    static constexpr int STAGE = 2 * TILE;          // K tile, then V tile
    static constexpr int R = 7;                     // ring stages: the tiles the waves are spread over, and those in flight
    static constexpr int F = 3;                     // tiles in flight
    static constexpr int SLOT = TILE / 2;           // per compute wave: 16 output rows on their way to memory
    static constexpr int SLOTS = R * STAGE;
    static constexpr int FLAGS = SLOTS + NWC * SLOT;  // int32: [0] tiles landed, [1 + w] first tile compute wave w may still read
    static constexpr int TOTAL = FLAGS + 64;
    static_assert(TOTAL <= 160 * 1024, "one workgroup may use the whole LDS of a compute unit, not more");
};

constexpr int BAND_MAX_COMPUTE_WAVES = 11;

// Blocks and tiles of one sequence of n rows under the window (left, right), both >= 0.
struct BandPlan {
    int n, left, right, n_tiles;
    __device__ __forceinline__ int first(int j) const { const int lo = 32 * j - left; return lo > 0 ? lo / KT : 0; }
    __device__ __forceinline__ int last(int j) const {
        int t_hi = 32 * j + 31;
        t_hi = t_hi < n - 1 ? t_hi : n - 1;
        const int64_t hi = (int64_t)t_hi + right;
        return (int)((hi < n - 1 ? hi : n - 1) / KT);
    }
};

// How long a wave polls an LDS word before it gives up (a few milliseconds): the waits below always end
// - the loader never waits for a tile that a compute wave still needs, see the kernel - and the bound only
// guarantees that a mistake in that reasoning would show as wrong numbers and not as a wave that never exits.
constexpr int BAND_SPIN_LIMIT = 1 << 16;

// One (sequence, head) of the launch as a wave sees it (all fields wave-uniform).
struct BandItem {
    int64_t row0;  // first row of the sequence in the packed tensors
    int n;         // its rows; <= 0: nothing to do (empty sequence, or padding of the item grid)
    int h;
};

template <int D, int NWC>
__global__ __launch_bounds__(64 * (NWC + 1), 1) void swa_band_fwd_kernel(AttnParams p, int n_items) {
    using SM = BandSmem<D, NWC>;
    using L = TileLayout<D>;
    constexpr int KC = D / 16, DB = D / 32;
    constexpr int TI = 2 * TileDma<D, 1, SWZ_K>::INSTR;  // load instructions of a key / value tile pair
    static_assert(SM::F == 3 && SM::F * TI < 64 && SM::R > SM::F, "tiles in flight: their loads must fit the vmcnt counter, their stages the ring");
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    // ---- the work items of this workgroup.  The launch is persistent (one workgroup per compute unit): workgroup w
    // of G takes the items w, 2G - 1 - w, 2G + w, 4G - 1 - w, ... of the list (sequences in scheduler order, longest
    // first; all heads of eight sequences, then the next eight) - on a list sorted by length the forward and the
    // backward sweep of every pair of rounds add up to nearly the same work for every workgroup.  Every wave walks
    // that list on its own with scalar loads, one item ahead, and the key tiles of ALL its items form one stream
    // with one running tile number: the loader goes on into the next item while the compute waves finish the
    // current one, so an item's first tiles are already in the ring when its first blocks start.
    const int G = gridDim.x;
    // (scalar loads: the lists are read-only for the whole kernel)
    const __attribute__((address_space(4))) int32_t* const order_c = (const __attribute__((address_space(4))) int32_t*)(uintptr_t)p.order;
    const __attribute__((address_space(4))) int32_t* const off_c = (const __attribute__((address_space(4))) int32_t*)(uintptr_t)p.kv_off;
    auto describe = [&](int k, BandItem& it) -> bool {
        const int64_t i = (int64_t)k * G + ((k & 1) ? G - 1 - (int)blockIdx.x : (int)blockIdx.x);
        if (i >= n_items) return false;
        const int slot = (int)(i & 7);
        const int64_t jj = i >> 3;
        it.h = (int)(jj % p.H);
        const int64_t e = (jj / p.H) * 8 + slot;
        it.row0 = 0;
        it.n = 0;
        if (e < p.B) {
            const int b = order_c ? order_c[e] : (int)e;
            it.row0 = off_c[b];
            it.n = off_c[b + 1] - (int)it.row0;
        }
        return true;
    };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const uint32_t lds0 = lds_address(lds);
    // (LDS address space kept in the type: a generic pointer would make every poll a flat memory operation)
    volatile __attribute__((address_space(3))) int* const flags = (volatile __attribute__((address_space(3))) int*)(lds + SM::FLAGS);

    // the words start at "nothing landed, nothing read"; the only barrier of the kernel orders that before any wait
    if (tid <= NWC) flags[tid] = 0;
    __syncthreads();

    if (wave == 0) {
        // ================= loader =================
        TileDma<D, 1, SWZ_K> kdma;
        TileDma<D, 1, SWZ_V> vdma;
        kdma.init(lane, 0, row_bytes);
        vdma.init(lane, 0, row_bytes);
        int T = 0;  // running tile number over all items of this workgroup
        BandItem cur, nxt;
        bool have = describe(0, cur);
        for (int k = 0; have; ++k) {
            const bool have_nxt = describe(k + 1, nxt);
            if (cur.n > 0) {
                const int n = cur.n;
                const int NT = (n + KT - 1) / KT;
                const char* K = (const char*)((const bf16_t*)p.k + (cur.row0 * p.H + cur.h) * D);
                const char* V = (const char*)((const bf16_t*)p.v + (cur.row0 * p.H + cur.h) * D);
                for (int t = 0; t < NT; ++t, ++T) {
                    // tiles T - F .. T - 1 are in flight: once T - F has landed it is published, before anything else, so
                    // that waves ahead of the others are not held up by the wait below
                    if (T >= SM::F) {
                        wait_vmcnt<(SM::F - 1) * TI>();
                        asm volatile("" ::: "memory");
                        if (lane == 0) flags[0] = T - SM::F + 1;
                    }
                    if (T >= SM::R) {
                        // the stage of tile T - R: every compute wave must be past that tile.  (It will be: a wave that is
                        // not has its tile in LDS already - tiles up to T - F have been published, F < R - and needs
                        // nothing from here.)
                        const int need = T - SM::R + 1;
                        for (int spin = 0; spin < BAND_SPIN_LIMIT; ++spin) {
                            const int prog = lane < NWC ? flags[1 + lane] : need;
                            if (__builtin_amdgcn_ballot_w64(prog < need) == 0) break;
                            __builtin_amdgcn_s_sleep(1);
                        }
                        asm volatile("" ::: "memory");  // the loads below stay behind the poll
                    }
                    const uint32_t dst = lds0 + (T % SM::R) * SM::STAGE;
                    kdma.issue(K + t * tile_bytes, n - t * KT, dst);
                    vdma.issue(V + t * tile_bytes, n - t * KT, dst + SM::TILE);
                }
            }
            cur = nxt;
            have = have_nxt;
        }
        // the last tiles land one by one
        if (T >= 3) { wait_vmcnt<2 * TI>(); asm volatile("" ::: "memory"); if (lane == 0) flags[0] = T - 2; }
        if (T >= 2) { wait_vmcnt<TI>(); asm volatile("" ::: "memory"); if (lane == 0) flags[0] = T - 1; }
        wait_vmcnt<0>();
        asm volatile("" ::: "memory");
        if (lane == 0) flags[0] = T;
        return;
    }

    // ================= compute waves =================
    const int cw = wave - 1;
    const int r = lane & 31, g = lane >> 5;
    const float sc = p.scale * LOG2E;
    const int k_rd = L::k_offset(r, g);
    const int v_rd = SM::TILE + L::v_offset(4 * g + ((lane & 15) >> 2), (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);

    bf16x8 qf[KC];
    f32x16 oacc[DB][1];
    float m_ref = -INFINITY, l_run = 0.f;
    int key_lo = 0x3fffffff;
    unsigned key_span = 0u;
    int nq = 0;  // queries of the current block
    int landed = 0;  // tiles of the stream that this wave has seen landed

    // B-operand fragments of block j of item `it` straight from global memory into the registers that hold them
    // (column = query r, contraction = channels 16*kc + 8g ..: lane (r, g) reads every second 16-byte chunk of its own
    // query row; rows past the end repeat the last one).  Issued while the previous block's last tile and output are
    // still in progress - the old fragments are dead after that tile's first contraction - so the round trip is hidden.
    auto load_query_fragments = [&](const BandItem& it, int j) {
        int lane_w = lane;
        asm volatile("" : "+v"(lane_w));  // address arithmetic in place, not kept in registers across the key loop
        const int rows = it.n - KT * j < KT ? it.n - KT * j : KT;
        const int rq = (lane_w & 31) < rows ? (lane_w & 31) : rows - 1;
        const bf16_t* src = (const bf16_t*)p.q + ((it.row0 + (int64_t)KT * j + rq) * p.H + it.h) * D + 8 * (lane_w >> 5);
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[kc] = *(const bf16x8*)(src + 16 * kc);
    };
    // Output rows of block j.  The lane holds query r, channels 32*db + 8*(v/4) + 4g + (v%4); the rows go out whole
    // (16 lanes x 16 bytes each), 16 rows at a time through the wave's LDS slot (16-byte chunks of a row XOR-swizzled
    // by the row).  (Stores of 32-byte pieces straight from registers were measured: 2.1 ms against 2.0 ms at the
    // bench size, and 2.9 ms with the non-temporal hint.)
    auto write_block = [&](const BandItem& it, int j) {
        int lane_w = lane;
        asm volatile("" : "+v"(lane_w));  // address arithmetic in place, not kept in registers across the key loop
        const int r = lane_w & 31, g = lane_w >> 5;
        constexpr int CHUNKS = D / 8;
        char* const slot = lds + SM::SLOTS + cw * SM::SLOT;
        const float l_tot = halves_sum(l_run);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const int64_t grow = it.row0 + (int64_t)KT * j;  // first row of the block in the packed tensors
        if (p.lse && g == 0 && r < nq)
            p.lse[(int64_t)it.h * p.total_q + grow + r] = l_tot > 0.f ? (m_ref + __builtin_amdgcn_logf(l_tot)) * (1.f / LOG2E) : -INFINITY;
        bf16_t* obase = (bf16_t*)p.o + grow * hd + (int64_t)it.h * D;
        constexpr int O_STORES = 16 * CHUNKS / 64;
        const int chunk = lane_w % CHUNKS, rsub = lane_w / CHUNKS;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if ((r >> 4) == half) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg) {
                        bf16x4 out;
#pragma unroll
                        for (int e4 = 0; e4 < 4; ++e4) out[e4] = (bf16_t)(oacc[db][0][4 * vg + e4] * inv);
                        *(bf16x4*)(slot + (r & 15) * SM::ROW + (((4 * db + vg) ^ (r & (CHUNKS - 1))) << 4) + 8 * g) = out;
                    }
            }
#pragma unroll
            for (int i = 0; i < O_STORES; ++i) {
                const int row = i * (64 / CHUNKS) + rsub;  // inside the half
                const u32x4 val = *(const u32x4*)(slot + row * SM::ROW + ((chunk ^ (row & (CHUNKS - 1))) << 4));
                if (16 * half + row < nq) __builtin_nontemporal_store(val, (u32x4*)(obase + (16 * half + row) * hd + chunk * 8));
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the slot has been read before the other half overwrites it
        }
    };
    // One key tile of the current block: tile s of the item, number T0 + s of the workgroup's stream.  On the block's
    // last tile the query fragments of the wave's next block (`pre_it`, `pre_j`; pre_j < 0: none) are requested as
    // soon as this tile's first contraction has consumed the current ones.
    // `fresh` (std::true_type on the block's first tile): the accumulators are assigned, not added to, and the running
    // softmax statistics are set, not updated - no zeroing of 64 registers per block, no rescaling of zeros.
    auto tile_step = [&](const BandItem& it, int T0, int jc, int s, const BandItem& pre_it, int pre_j, auto fresh) {
        constexpr bool FRESH = decltype(fresh)::value;
        const int n = it.n;
        const int gs = T0 + s;
        // tile gs has landed?  (the count last seen is kept: the loader is usually several tiles ahead, and the LDS
        // round trip of a poll is then saved; the branch is uniform)
        if (landed <= gs) {
            for (int spin = 0; spin < BAND_SPIN_LIMIT; ++spin) {
                landed = __builtin_amdgcn_readfirstlane(flags[0]);
                if (landed > gs) break;
                __builtin_amdgcn_s_sleep(1);
            }
        }
        asm volatile("" ::: "memory");  // the tile reads below stay behind the poll
        const char* st = lds + (gs % SM::R) * SM::STAGE;
        // ---- S^T = K Q^T
        f32x16 sacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 a = *(const bf16x8*)(st + (k_rd ^ (kc << 5)));
            sacc = mfma32(a, qf[kc], sacc);
        }
        if (pre_j >= 0) load_query_fragments(pre_it, pre_j);
        // ---- online softmax; only tiles that some query of the block sees partly take the masked path
        const int key_base = s * KT;
        const int tq_lo = KT * jc, tq_hi = KT * jc + nq - 1;
        bool need_mask = key_base + KT > n || nq < KT;
        if (key_base < tq_hi - p.left) need_mask = true;
        if ((int64_t)key_base + KT - 1 > (int64_t)tq_lo + p.right) need_mask = true;
        bf16x8 pf[2];
        score_to_weights<KUNLUN_ACT_SOFTMAX, DB, 1, FRESH>(sacc, need_mask, (unsigned)(key_base + 4 * g - key_lo), key_span, sc, m_ref,
                                                           l_run, oacc, 0, pf);
        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const char* src = st + (v_rd ^ (db << 6)) + c * 16 * SM::ROW;
                const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src));
                const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src + 8 * SM::ROW));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const bf16x8 a = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
                if (FRESH && c == 0) {
                    f32x16 zero;
#pragma unroll
                    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                    oacc[db][0] = mfma32(a, pf[c], zero);
                } else {
                    oacc[db][0] = mfma32(a, pf[c], oacc[db][0]);
                }
            }
        }
        // every LDS read of the tile has been issued (the LDS serves a wave's operations in order, and the empty
        // statement keeps the compiler from moving the store up): publish
        asm volatile("" ::: "memory");
        if (lane == 0) flags[1 + cw] = gs + 1;
    };

    int T0 = 0;             // stream number of the current item's first tile
    bool q_ready = false;   // the fragments of this wave's first block of the current item were requested during the item before
    BandItem cur, nxt;
    bool have = describe(0, cur);
    for (int k = 0; have; ++k) {
        const bool have_nxt = describe(k + 1, nxt);
        if (cur.n > 0) {
            const int n = cur.n;
            BandPlan plan;
            plan.n = n; plan.left = p.left; plan.right = p.right; plan.n_tiles = (n + KT - 1) / KT;
            const int NB = plan.n_tiles;  // query blocks = key tiles
            // this wave's blocks: cw, cw + NWC, ...
            if (cw < NB && !q_ready) load_query_fragments(cur, cw);
            q_ready = false;
            for (int jc = cw; jc < NB; jc += NWC) {
                const int fj = plan.first(jc), ej = plan.last(jc);
                // from here on this wave reads no tile before fj
                if (lane == 0) flags[1 + cw] = T0 + fj;
                m_ref = -INFINITY; l_run = 0.f;
                nq = n - KT * jc;
                nq = nq > KT ? KT : nq;
                {
                    const int tq = KT * jc + r;  // this lane's query (inside the sequence)
                    int lo = tq - p.left, hi = n - 1;
                    lo = lo > 0 ? lo : 0;
                    if ((int64_t)tq + p.right < hi) hi = tq + p.right;
                    const bool empty = hi < lo || r >= nq;
                    key_lo = empty ? 0x3fffffff : lo;
                    key_span = empty ? 0u : (unsigned)(hi - lo);
                }
                // the block after this one: in this item, else the wave's first block of the next item (if it has one)
                const bool same = jc + NWC < NB;
                q_ready = !same && have_nxt && nxt.n > KT * cw;
                const BandItem pre = same ? cur : nxt;
                const int pre_j = same ? jc + NWC : (q_ready ? cw : -1);
                if (fj < ej) {
                    tile_step(cur, T0, jc, fj, cur, -1, std::true_type{});
                    for (int s = fj + 1; s < ej; ++s) tile_step(cur, T0, jc, s, cur, -1, std::false_type{});
                    tile_step(cur, T0, jc, ej, pre, pre_j, std::false_type{});
                } else {
                    tile_step(cur, T0, jc, ej, pre, pre_j, std::true_type{});
                }
                write_block(cur, jc);
            }
            T0 += NB;
            // done with this item: this wave holds back none of its stages
            if (lane == 0) flags[1 + cw] = T0;
        }
        cur = nxt;
        have = have_nxt;
    }
    // no further item
    if (lane == 0) flags[1 + cw] = 0x7fffffff;
}

// The window must be bounded on both sides and narrow enough for the compute waves of one workgroup:
// c_l + c_r + 2 <= BAND_MAX_COMPUTE_WAVES (see the header of this file).
static int band_compute_waves(int left, int right) {
    if (left < 0 || right < 0) return 0;
    const int64_t c_l = ((int64_t)left + 31) / 32, c_r = ((int64_t)right + 31) / 32;
    const int64_t need = c_l + c_r + 2;
    if (need > BAND_MAX_COMPUTE_WAVES || c_l + c_r + 2 > BAND_MAX_COMPUTE_WAVES) return 0;
    return (int)need;
}

// Worth it when the window keeps most waves of a compute unit busy (wide enough) and the launch has enough
// (sequence, head) items for one workgroup per compute unit to balance (one item at a time per compute unit;
// measured down to two items per compute unit: 139 against 164 us on 512 sequences of 256..2048 rows).
bool swa_band_applies(const AttnParams& p) {
    const int nwc = band_compute_waves(p.left, p.right);
    return p.windowed && nwc >= 8 && (int64_t)p.B * p.H >= 2 * 256 && (p.d == 128 || p.d == 64 || p.d == 32) && p.scale > 0.f;
}

template <int D, int NWC>
static hipError_t launch_band(const AttnParams& p, hipStream_t stream) {
    constexpr int bytes = BandSmem<D, NWC>::TOTAL;
    auto kern = swa_band_fwd_kernel<D, NWC>;
    if (bytes > 64 * 1024) {
        // once per process (thread-safe initialisation of a function-local static); not a stream operation
        static const hipError_t raised = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (raised != hipSuccess) return raised;
    }
    const int64_t n_items = (((int64_t)p.B + 7) / 8) * 8 * p.H;
    const int64_t resident = compute_units();  // one workgroup (all of the LDS) per compute unit
    const unsigned grid = (unsigned)(n_items < resident ? n_items : resident);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * (NWC + 1)), bytes, stream, p, (int)n_items);
    return hipGetLastError();
}

// p.order: the sequences, longest first (written by the scheduler kernel), or null.
hipError_t launch_swa_band_fwd(const AttnParams& p, hipStream_t stream) {
    const int nwc = band_compute_waves(p.left, p.right);
    // two workgroup sizes: up to 9 or up to 11 compute waves (a wave without a block only passes the barriers)
    if (nwc <= 9)
        return p.d == 128 ? launch_band<128, 9>(p, stream) : p.d == 64 ? launch_band<64, 9>(p, stream) : launch_band<32, 9>(p, stream);
    return p.d == 128 ? launch_band<128, 11>(p, stream) : p.d == 64 ? launch_band<64, 11>(p, stream) : launch_band<32, 11>(p, stream);
}

}  // namespace kunlun
