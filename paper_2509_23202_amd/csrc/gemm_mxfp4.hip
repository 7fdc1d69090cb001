// MXFP4 W4A4 GEMM on the CDNA4 block-scaled FP4 MFMA (arXiv 2509.23202, Section 4.2 item 2: the FP4 matmul
// Q(W H) Q(X H)^T with hardware-applied group scales).
//
//   out[m,n] = sum_k  2^(sa[m,k/32]-127) * 2^(sw[n,k/32]-127) * a[m,k] * w[n,k]
//
// v_mfma_scale_f32_16x16x128_f8f6f4 multiplies a 16x128 by a 128x16 FP4 tile; every lane supplies 32 consecutive
// K-elements of one row (16 bytes) and one E8M0 byte that scales exactly those 32 elements -- the MXFP4 group.
// Both operands arrive in "GEMM layout": 1 KB fragments already in lane order (layout.hpp), so a fragment moves
// global -> LDS with one 16-byte direct-to-LDS load per lane and LDS -> registers with one conflict-free
// ds_read_b128 per lane; no re-layout pass runs between the quantizer and the GEMM.  (Direct-to-LDS loads write
// lane l's bytes at LDS base + 16*l, which is exactly the fragment order.)
//
// Roles are swapped on purpose: the W fragment is the MFMA's A operand (rows = n) and the X fragment its B
// operand (columns = m).  A lane then owns four consecutive n of one m, i.e. one 8-byte bf16x4 store.
//
// Block tile BM x BN, K-step 128, STAGES-deep LDS ring fed by direct-to-LDS loads (tracked with vmcnt), one
// barrier per K-step.  Scales take the same route into a single LDS buffer: with four and more stages one 16-byte
// copy per pair of row-blocks and 8 K-steps, with three stages one 4-byte copy per row-block and 4 K-steps.
#include "device_util.hpp"
#include "internal.hpp"
#include "layout.hpp"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <type_traits>

namespace fp4mr {
namespace {

struct GemmArgs {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* w_codes;
    const uint8_t* w_scales;
    void* out;
    int64_t M, N, K;
    int tiles_m, tiles_n;
    float alpha;  // factor on the result: powers of 4/3 for operands whose scales carry the tensor-level 4/3, else 1
    int split_steps;  // split-K launches: K-steps per split (a multiple of 8); blockIdx.y is the split, out the fp32 partials
};

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);  // expcnt / lgkmcnt: no wait
}

// Barrier without the memory fence of __syncthreads(): a fence would make the compiler drain every outstanding
// load (vmcnt(0)) and with it the whole prefetch ring.  The data hazards are handled explicitly instead: the
// wait_vmcnt above it covers this wave's direct-to-LDS copies, the barrier publishes them to the other waves.
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ void wait_lgkmcnt0()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0); vmcnt / expcnt: no wait
}

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

template <int OPSEL>
__device__ __forceinline__ v4f mfma_fp4(const v4i& a, const v4i& b, const v4f& c, uint32_t sa, uint32_t sb)
{
    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
    const v8i b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    // cbsz = blgp = 4: both operands E2M1.  op_sel picks byte OPSEL of each scale register.
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, c, 4, 4, OPSEL, (int)sa, OPSEL, (int)sb);
}

__device__ __forceinline__ void remap_block(int bid, int nblocks, int tiles_m, int tiles_n, int& tm, int& tn)
{
    // Workgroups are dealt round-robin to the 8 XCDs.  Give every XCD one contiguous range of logical tile
    // ids, and order logical ids in bands of GM tile-rows, so the tiles that share an L2 share operands.
    const int per = nblocks >> 3, rem = nblocks & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    const int L = (xcd < rem) ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    constexpr int GM = 4;
    const int band = GM * tiles_n;
    const int gidx = L / band;
    const int first_m = gidx * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_band = L - gidx * band;
    tm = first_m + in_band % gsz;
    tn = in_band / gsz;
}

// Four-wave workgroups with a three-stage ring are sized so that two of them share a compute unit (registers: 256 per
// wave; LDS: under 80 KB): while one converts and stores its tile the other keeps the matrix pipes busy.
template <int BM, int BN, int WM, int WN, int STAGES>
constexpr int kWgsPerCu = ((BM / WM) * (BN / WN) == 4 && STAGES == 3) ? 2 : 1;

template <int BM, int BN, int WM, int WN, int STAGES, bool OUT_F32, int RD = 2, bool PERSIST = false, bool SPLITK = false>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) __attribute__((amdgpu_waves_per_eu(kWgsPerCu<BM, BN, WM, WN, STAGES>)))
void gemm_mx_kernel(GemmArgs g)
{
    constexpr int NWM = BM / WM, NWN = BN / WN, NW = NWM * NWN;
    constexpr int FX = BM / 16, FW = BN / 16, F = FX + FW;  // fragments per stage
    constexpr int LPW = (F + NW - 1) / NW;                  // fragment loads per wave per stage
    constexpr int TM = WM / 16, TN = WN / 16;               // MFMA tiles per wave
    constexpr int STAGE_BYTES = F * 1024;
    static_assert(STAGES >= 3 && STAGES <= 8, "ring bookkeeping is written for 3 to 8 stages");

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int lane = threadIdx.x & 63;
    // the wave index is uniform across the wavefront: telling the compiler keeps every fragment base address,
    // LDS offset and tile coordinate in scalar registers (the vector file is needed for accumulators and fragments)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wm = wave % NWM, wn = wave / NWM;
    const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)lane * 4u;

    // PERSIST: the grid is one workgroup per compute unit and a workgroup walks the tiles blockIdx.x,
    // blockIdx.x + gridDim.x, ...; otherwise the grid has one workgroup per tile and the loop below runs once.
    const int ntiles = g.tiles_m * g.tiles_n;
    int tile = blockIdx.x;

    const int64_t KC = g.K >> 7;            // K-steps (of a row-block in memory)
    const int64_t KS = (g.K + 511) >> 9;    // scale super-steps (likewise)
    // SPLITK: this workgroup multiplies K-steps kt0 .. kt0 + KT - 1 only (kt0 a multiple of 8: whole scale batches) and
    // writes its fp32 partial tile to slice blockIdx.y of the output, which a reduction kernel adds up in split order
    static_assert(!SPLITK || (OUT_F32 && !PERSIST), "split-K workgroups write fp32 partials, one tile each");
    const int kt0 = SPLITK ? (int)blockIdx.y * g.split_steps : 0;
    const int KT = SPLITK ? min(g.split_steps, (int)KC - kt0) : (int)KC;
    const int KS_rem = (int)KS - (kt0 >> 2);  // scale blocks from kt0 to the end of K

    // Operands are addressed through buffer resources: one VGPR (16 * lane) is the only per-lane address and every
    // fragment's position is a scalar offset.  Row-blocks past the end of an operand (last tile) are clamped to its
    // last row-block: the duplicates only feed output rows / columns that are never stored.
    const int a_rbs = (int)((g.M + 15) / 16), w_rbs = (int)((g.N + 15) / 16);
    auto make_rsrc = [](const uint8_t* base, int64_t bytes) {
        const uint32_t n = bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, (int)n, 0x00020000);
    };
    // bases at the tile's first row-block keep every scalar offset far below 2^31
    int tm, tn;                  // tile whose operands the loads below address
    __amdgpu_buffer_rsrc_t rs_ac, rs_wc, rs_as, rs_ws;
    int a_rb_last, w_rb_last;    // largest valid row-block relative to the base
    auto set_tile = [&](int t) {
        remap_block(t, ntiles, g.tiles_m, g.tiles_n, tm, tn);
        const int a_rb0 = min(tm * FX, a_rbs - 1), w_rb0 = min(tn * FW, w_rbs - 1);
        const int64_t c0 = (int64_t)kt0 * 1024, s0 = (int64_t)(kt0 >> 2) * 256;  // (0 unless SPLITK)
        rs_ac = make_rsrc(g.a_codes + (int64_t)a_rb0 * KC * 1024 + c0, (int64_t)(a_rbs - a_rb0) * KC * 1024 - c0);
        rs_wc = make_rsrc(g.w_codes + (int64_t)w_rb0 * KC * 1024 + c0, (int64_t)(w_rbs - w_rb0) * KC * 1024 - c0);
        rs_as = make_rsrc(g.a_scales + (int64_t)a_rb0 * KS * 256 + s0, (int64_t)(a_rbs - a_rb0) * KS * 256 - s0);
        rs_ws = make_rsrc(g.w_scales + (int64_t)w_rb0 * KS * 256 + s0, (int64_t)(w_rbs - w_rb0) * KS * 256 - s0);
        a_rb_last = a_rbs - 1 - a_rb0;
        w_rb_last = w_rbs - 1 - w_rb0;
    };
    set_tile(tile);

    // Scales: every (row-block, 4 K-steps) owns 256 bytes = one dword per lane.  They travel global -> LDS with
    // direct-to-LDS loads (so no VGPR is ever the target of an in-flight load inside the main loop) and are read back
    // once per 4 K-steps.
    //   SC8 (four and more stages): a batch is 8 K-steps.  One 16-byte-per-lane copy fetches 512 bytes (two
    //   consecutive 4-step blocks) of TWO row-blocks -- lanes 0..31 the first, lanes 32..63 the second; the address is
    //   per lane, the LDS side is base + 16 * lane -- so a workgroup needs (FX + FW) / 2 copies per 8 K-steps instead of
    //   2 * (FX + FW) four-byte ones.  The vector-memory path is a co-limiter of this loop (extra address traffic
    //   measured far more expensive than its bytes), which is what this saves.  One buffer: the batch of steps
    //   8b+8 .. 8b+15 is requested in step 8b+4, after every wave has read the second half of batch b into registers
    //   (end of step 8b+3, then that step's barrier), and it has landed before the read at the end of step 8b+7
    //   (loads complete in order, and step 8b+7 has waited for the stage requested in step 8b+5).
    //   Otherwise (three stages): 4-byte copies, a batch is 4 K-steps.
    constexpr bool SC8 = STAGES >= 4;
    constexpr int XP = (FX + 1) / 2, WP = (FW + 1) / 2;    // pairs of row-blocks
    constexpr int NS = SC8 ? (XP + WP + NW - 1) / NW : LPW; // scale loads per wave per batch
    constexpr int SCALE_BYTES = SC8 ? (XP + WP) * 1024 : F * 256;
    static_assert(NS <= LPW, "a scale load is issued in front of a fragment load of the same step");
    // One scale buffer up to five stages.  From six stages on the stage a step waits for was requested more than four steps
    // earlier, so a batch requested in step 8b+4 would no longer be covered by the wait of step 8b+7 (loads complete in
    // issue order: a wait for stage kt+1 covers what was requested before it): the batch is then requested in step 8b+0,
    // into the other of TWO buffers (the one whose batch was last read at the end of step 8b-5).
    constexpr int SD = (SC8 && STAGES >= 6) ? 2 : 1;
    char* const scale_ring = smem + STAGES * STAGE_BYTES;
    const int kc_bytes = (int)KC * 1024, ks_bytes = (int)KS * 256;

    v4f acc[TN][TM];
    uint32_t sx[TM], sw[TN];
    // Software pipeline of the LDS reads: the X fragments of step kt+1 are read into the other half of xf[2][.]
    // while step kt computes, and the W fragments run through a 4-deep register ring two groups of TM MFMAs ahead
    // of their use -- so no MFMA waits on LDS latency, at a cost of 2*TM*4 + 16 fragment registers.
    // W-fragment register ring; RD = how many MFMA groups ahead it is filled (three slots when TN is not a multiple of 4)
    constexpr int RING = (TN % 4 != 0) ? 3 : ((RD <= 3) ? 4 : 8);
    v4i xf[2][TM], wring[RING];
    static_assert(TN % RING == 0 && RD < RING && RD <= TN, "the W-fragment ring index must be static");
    // every wave issues exactly LPW fragment loads per stage and NS scale loads per batch so that the vmcnt
    // bookkeeping is uniform; when F is not a multiple of NW the spare slots re-copy the last fragment (same bytes
    // to the same place)
    // which operand load slot i of this wave belongs to: known at compile time (i is a constant after unrolling)
    // whenever the X fragments divide evenly among the waves, which keeps the step body free of branches
    auto is_x = [&](int f, int i) { return (FX % NW == 0) ? (i < FX / NW) : (f < FX); };
    auto issue_scale_one = [&](int ss, int i) {
        if constexpr (SC8) {
            // ss = the batch: 4-step blocks 2 * ss and 2 * ss + 1 (past the end: the last block again; what lies behind it
            // in the 512 bytes is never used, and reads beyond the operand return zeros)
            const int blk = min(2 * ss, KS_rem - 1);
            const int p = min(wave + i * NW, XP + WP - 1);
            const uint32_t half = (uint32_t)lane >> 5, col = ((uint32_t)lane & 31u) * 16u;
            if ((XP % NW == 0) ? (i < XP / NW) : (p < XP)) {
                const uint32_t rb = (uint32_t)min(2 * p + (int)half, a_rb_last);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_as, (lds_void*)(scale_ring + (SD == 2 ? (ss & 1) * SCALE_BYTES : 0) + p * 1024), 16, rb * (uint32_t)ks_bytes + col, blk * 256, 0, 0);
            } else {
                const uint32_t rb = (uint32_t)min(2 * (p - XP) + (int)half, w_rb_last);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_ws, (lds_void*)(scale_ring + (SD == 2 ? (ss & 1) * SCALE_BYTES : 0) + p * 1024), 16, rb * (uint32_t)ks_bytes + col, blk * 256, 0, 0);
            }
            return;
        }
        char* base = scale_ring;
        ss = ss < KS_rem ? ss : KS_rem - 1;  // the batch past the end re-reads the last one
        const int f = min(wave + i * NW, F - 1);
        if (is_x(f, i)) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_as, (lds_void*)(base + f * 256), 4, lane4, min(f, a_rb_last) * ks_bytes + ss * 256, 0, 0);
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_ws, (lds_void*)(base + f * 256), 4, lane4, min(f - FX, w_rb_last) * ks_bytes + ss * 256, 0, 0);
    };
    auto issue_frag_one = [&](int kt, char* base, int i) {
        const int f = min(wave + i * NW, F - 1);
        if (is_x(f, i)) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_ac, (lds_void*)(base + f * 1024), 16, lane16, min(f, a_rb_last) * kc_bytes + kt * 1024, 0, 0);
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wc, (lds_void*)(base + f * 1024), 16, lane16, (min(f - FX, w_rb_last)) * kc_bytes + kt * 1024, 0, 0);
    };
    auto issue_scales = [&](int ss) {
#pragma unroll
        for (int i = 0; i < NS; ++i) issue_scale_one(ss, i);
    };
    auto read_scales = [&](int64_t ss, uint32_t (&dx)[TM], uint32_t (&dw)[TN]) {  // ss = 4-step block
        if constexpr (SC8) {
            // a row-block's 512 bytes: even block, odd block (two buffers: batch ss / 2 is in buffer (ss / 2) % 2)
            const char* base = scale_ring + (SD == 2 ? (int)((ss >> 1) & 1) * SCALE_BYTES : 0) + (ss & 1) * 256;
#pragma unroll
            for (int j = 0; j < TM; ++j) dx[j] = *(reinterpret_cast<const uint32_t*>(base + (wm * TM + j) * 512) + lane);
#pragma unroll
            for (int i = 0; i < TN; ++i) dw[i] = *(reinterpret_cast<const uint32_t*>(base + (2 * XP + wn * TN + i) * 512) + lane);
        } else {
            const char* base = scale_ring;
#pragma unroll
            for (int j = 0; j < TM; ++j) dx[j] = *(reinterpret_cast<const uint32_t*>(base + (wm * TM + j) * 256) + lane);
#pragma unroll
            for (int i = 0; i < TN; ++i) dw[i] = *(reinterpret_cast<const uint32_t*>(base + (FX + wn * TN + i) * 256) + lane);
        }
    };
    auto read_x = [&](int kt, auto ptag, int j) {
        constexpr int P = decltype(ptag)::value;
        xf[P][j] = *(reinterpret_cast<const v4i*>(smem + (kt % STAGES) * STAGE_BYTES + (wm * TM + j) * 1024) + lane);
    };
    auto read_w = [&](int kt, int i) {  // into ring slot i % 4 (i is a compile-time constant after unrolling)
        wring[i % RING] = *(reinterpret_cast<const v4i*>(smem + (kt % STAGES) * STAGE_BYTES + (FX + wn * TN + i) * 1024) + lane);
    };

    // prologue of a tile: scales of super-step 0 and STAGES-1 stages on their way into ring slots 0 .. STAGES-2
    auto issue_prologue = [&]() {
        issue_scales(0);
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s) {
#pragma unroll
            for (int i = 0; i < LPW; ++i) issue_frag_one(min(s, KT - 1), smem + s * STAGE_BYTES, i);
        }
    };
    issue_prologue();
    wait_vmcnt<(STAGES - 2) * LPW>();

    // One K-step.  J = kt % 8 (SC8) or kt % 4: J & 3 selects the scale byte (op_sel), J & 1 the X register half.
    //   top:    stage kt+1 must have landed (this wave's copies: vmcnt; everybody's: barrier).  The same barrier
    //           says that every wave is done reading stage kt-1, whose LDS buffer is refilled with stage kt+STAGES-1.
    //   vmcnt:  allowed in flight = the STAGES-3 stages after kt+1, plus one scale batch when it was issued after
    //           stage kt+1's loads (batches go out at J == 0, ahead of that step's fragment loads).
    constexpr int NST = TM * (16 * (WN / 8) / 64);  // store instructions a wave issues for one interior output tile
    static_assert((STAGES - 2) * LPW + NST < 64 && (STAGES - 3) * LPW + NS + NST < 64, "vmcnt is a 6-bit counter");
    bool pend = false;  // persistent workgroups: the previous tile's stores may be outstanding at the top of this tile
    constexpr int XPG = (TM + TN - 1) / TN;  // X-fragment reads folded in front of each group of TM MFMAs
    // The LDS reads for "the next step" are unconditional: in the very last step they fetch stale bytes of the ring
    // that nothing consumes, which keeps the step body free of branches (and of a second copy of the code).
    auto step = [&](int kt, auto jtag, auto wtag) {
        constexpr int J = decltype(jtag)::value;
        constexpr int SKEW = (2 * decltype(wtag)::value) % TM;  // MFMA index inside a group after which this wave issues its loads
        constexpr int P = J & 1;
        constexpr int JB = (SC8 && SD == 1) ? 4 : 0;  // the step of a period that requests the next scale batch
        constexpr int PER = SC8 ? 8 : 4;                // steps per scale batch
        // the batch was requested 1 .. STAGES - 3 steps ago, i.e. behind the loads of the stage this step waits for
        constexpr bool batch_after = ((J - JB - 1 + PER) % PER) <= STAGES - 4;
        constexpr int ALLOWED = (STAGES - 3) * LPW + (batch_after ? NS : 0);
        if constexpr (PERSIST && J <= STAGES - 3) {
            // first steps of a follow-on tile, as long as the stage they wait for (kt + 1) is one of the STAGES - 1 that
            // were prefetched: the previous tile's NST output stores were issued after those and may still be in flight
            // (vector memory operations complete in issue order, so the stages in front of the stores can be waited for
            // without waiting for the stores)
            if (pend && kt <= STAGES - 3) wait_vmcnt<ALLOWED + NST>(); else wait_vmcnt<ALLOWED>();
        } else {
            wait_vmcnt<ALLOWED>();
        }
        wait_lgkmcnt0();
        block_barrier();
        // The global -> LDS loads of stage kt+STAGES-1 (and, at J == 0, of the next scale batch) are spread over the
        // groups of MFMAs: a wave issues in order, and a burst of vector-memory instructions at the top of the step
        // would hold its MFMAs back while the CU's single address unit works through all four waves' bursts.
        // Past the last stage the loads re-copy stage KT-1 into a ring slot nobody reads any more: the step body stays
        // free of branches (which would let the compiler pull the MFMAs away from the loads they are meant to cover)
        // and the vmcnt bookkeeping needs no special case for the tail.
        const int kt_load = min(kt + STAGES - 1, KT - 1);
        char* const load_base = smem + ((kt + STAGES - 1) % STAGES) * STAGE_BYTES;
        constexpr int DPG = (LPW + TN - 1) / TN;  // loads per group
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            // W fragment two groups ahead (wraps into the next step), X fragments of the next step
            if (i + RD < TN) read_w(kt, i + RD);
            else read_w(kt + 1, i + RD - TN);
#pragma unroll
            for (int j = i * XPG; j < (i + 1) * XPG && j < TM; ++j) read_x(kt + 1, std::integral_constant<int, 1 - P>{}, j);
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                acc[i][j] = mfma_fp4<(J & 3)>(wring[i % RING], xf[P][j], acc[i][j], sw[i], sx[j]);
                if (j == SKEW) {
                    // the four waves of a workgroup run in lockstep (one barrier per step); issuing their loads at
                    // different points of the group keeps them from queueing up behind each other at the CU's one
                    // address unit while their MFMA pipes run dry
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int d = i * DPG; d < (i + 1) * DPG && d < LPW; ++d) {
                        if constexpr (J == JB) {
                            if (d < NS) issue_scale_one(SC8 ? (kt >> 3) + 1 : (kt >> 2) + 1, d);
                        }
                        issue_frag_one(kt_load, load_base, d);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // keep the instruction scheduler from hoisting the later groups' LDS reads up here: that would rebuild a
            // full second copy of the W fragments in registers
            __builtin_amdgcn_sched_barrier(0);
        }
        // scales of the next four steps (their batch landed before this step's barrier)
        if constexpr ((J & 3) == 3) read_scales((kt >> 2) + 1, sx, sw);
    };

    auto main_loop = [&](auto wtag) {
        for (int kt0 = 0; kt0 < KT; kt0 += (SC8 ? 8 : 4)) {
            step(kt0, std::integral_constant<int, 0>{}, wtag);
            if (kt0 + 1 < KT) step(kt0 + 1, std::integral_constant<int, 1>{}, wtag);
            if (kt0 + 2 < KT) step(kt0 + 2, std::integral_constant<int, 2>{}, wtag);
            if (kt0 + 3 < KT) step(kt0 + 3, std::integral_constant<int, 3>{}, wtag);
            if constexpr (SC8) {
                if (kt0 + 4 < KT) step(kt0 + 4, std::integral_constant<int, 4>{}, wtag);
                if (kt0 + 5 < KT) step(kt0 + 5, std::integral_constant<int, 5>{}, wtag);
                if (kt0 + 6 < KT) step(kt0 + 6, std::integral_constant<int, 6>{}, wtag);
                if (kt0 + 7 < KT) step(kt0 + 7, std::integral_constant<int, 7>{}, wtag);
            }
        }
    };

    // The epilogue transposes 16 output rows of the wave tile at a time through a staging area in the last ring
    // slot; the other slots are free for the next tile's prologue loads while the stores drain.
    constexpr int CPR = WN / 8;                  // 16-byte chunks per staged row
    constexpr int STAGING = 16 * WN * 2;         // bytes per wave
    constexpr bool STAGED = !OUT_F32 && NW * STAGING <= STAGE_BYTES && (CPR == 8 || CPR == 12 || CPR == 16);
    constexpr int SWZ = (CPR == 12) ? 3 : CPR - 1;  // chunk swizzle mask: XOR stays inside an aligned group of SWZ + 1 chunks

    for (;;) {
        // stage 0 and the first scale batch have landed (this wave's copies: the vmcnt wait before this point)
        block_barrier();
        read_scales(0, sx, sw);
#pragma unroll
        for (int j = 0; j < TM; ++j) read_x(0, std::integral_constant<int, 0>{}, j);
#pragma unroll
        for (int i = 0; i < RD; ++i) read_w(0, i);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

        if constexpr (SC8) {
            // (the eight-step period doubles the loop body: one copy of it, every wave issuing its loads at the same
            // point of an MFMA group; the per-wave skew below measured within noise)
            main_loop(std::integral_constant<int, 0>{});
        } else {
            switch (wave & 3) {
                case 0: main_loop(std::integral_constant<int, 0>{}); break;
                case 1: main_loop(std::integral_constant<int, 1>{}); break;
                case 2: main_loop(std::integral_constant<int, 2>{}); break;
                default: main_loop(std::integral_constant<int, 3>{}); break;
            }
        }
        wait_vmcnt<0>();  // the clamped loads of the last steps
        wait_lgkmcnt0();
        block_barrier();  // every wave is done with the operand ring, and nothing is in flight into it

        const int64_t m0 = (int64_t)tm * BM + wm * WM, n0 = (int64_t)tn * BN + wn * WN;  // this wave's output tile
        const bool interior = (int64_t)(tm + 1) * BM <= g.M && (int64_t)(tn + 1) * BN <= g.N;  // no lane is masked off
        const int next = tile + (int)gridDim.x;
        const bool more = PERSIST && next < ntiles;
        pend = false;
        if (more) {
            // the next tile's first stages travel while this tile's results are converted and stored
            set_tile(next);
            issue_prologue();
        }

        // A lane owns out[m][n..n+3] with m = m0 + 16*j + lane%16, n = n0 + 16*i + 4*(lane/16): stored directly that
        // is 16 rows x 32 bytes per instruction.  For bf16 output the rows go through LDS first so that every store
        // instruction writes 16 bytes per lane in whole rows.  A staged row is WN*2 bytes with its 16-byte chunks
        // XOR-swizzled by the row number: the 8-byte writes of a half-wave and the 16-byte reads of a quarter-wave
        // then both spread over all banks.
        // the lane-dependent address arithmetic of the epilogue is tied to a value defined here, so that the compiler
        // cannot hoist it above the tile loop and carry it (in registers the main loop needs) through every K-step
        int el = lane;
        asm volatile("" : "+v"(el));
        if (g.alpha != 1.0f) {
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) acc[i][j] *= g.alpha;
        }
        if (STAGED && (g.N & 7) == 0) {
            char* const mine = smem + (STAGES - 1) * STAGE_BYTES + wave * STAGING;
            typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
            const int wr = el & 15, wq = el >> 4;
#pragma unroll
            for (int j = 0; j < TM; ++j) {
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    const v4f v = acc[i][j];
                    const v4bf p = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
                    const int ch = (2 * i + (wq >> 1)) ^ (wr & SWZ);
                    *reinterpret_cast<v4bf*>(mine + wr * (WN * 2) + ch * 16 + (wq & 1) * 8) = p;
                }
#pragma unroll
                for (int it = 0; it < 16 * CPR / 64; ++it) {
                    const int c = it * 64 + el;
                    const int row = c / CPR, ch = c % CPR;
                    const v4i v = *reinterpret_cast<const v4i*>(mine + row * (WN * 2) + ((ch ^ (row & SWZ)) * 16));
                    const int64_t m = m0 + 16 * j + row, n = n0 + ch * 8;
                    // an interior tile issues exactly NST stores per wave (what the follow-on tile's vmcnt allowance counts)
                    if (interior || (m < g.M && n < g.N)) __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(static_cast<__bf16*>(g.out) + m * g.N + n));
                }
            }
            pend = more && interior;
        } else {
            // direct stores (fp32 output, or N not a multiple of 8)
            const int64_t m_base = m0 + (el & 15);
            const int64_t n_base = n0 + (el >> 4) * 4;
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int64_t m = m_base + 16 * j;
                if (m >= g.M) continue;
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    const int64_t n = n_base + 16 * i;
                    if (n >= g.N) continue;
                    const v4f v = acc[i][j];
                    if constexpr (OUT_F32) {
                        float* o = static_cast<float*>(g.out) + (SPLITK ? (int64_t)blockIdx.y * g.M * g.N : 0) + m * g.N + n;
                        if (n + 3 < g.N && (g.N & 3) == 0) {
                            *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
                        } else {
                            for (int e = 0; e < 4; ++e)
                                if (n + e < g.N) o[e] = v[e];
                        }
                    } else {
                        __bf16* o = static_cast<__bf16*>(g.out) + m * g.N + n;
                        typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
                        if (n + 3 < g.N && (g.N & 3) == 0) {
                            v4bf p = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
                            *reinterpret_cast<v4bf*>(o) = p;
                        } else {
                            for (int e = 0; e < 4; ++e)
                                if (n + e < g.N) o[e] = (__bf16)v[e];
                        }
                    }
                }
            }
        }
        if (!more) break;
        tile = next;
        // Stage 0 and the scale batch of the next tile were issued before this tile's stores: after an interior tile
        // (exact store count) wait for them only and let the stores drain under the first K-steps; otherwise wait for
        // everything.
        if (pend) wait_vmcnt<(STAGES - 2) * LPW + NST>(); else wait_vmcnt<0>();
    }
}


// out[i] = alpha * (partial[0][i] + partial[1][i] + ...), the splits added in their order (deterministic), as bf16 or fp32
template <bool OUT_F32>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int64_t mn, float alpha, void* out)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < mn; i += (int64_t)gridDim.x * 256) {
        float s = partial[i];
        for (int p = 1; p < splits; ++p) s += partial[(int64_t)p * mn + i];
        s *= alpha;
        if constexpr (OUT_F32) static_cast<float*>(out)[i] = s;
        else static_cast<__bf16*>(out)[i] = (__bf16)s;
    }
}

// the tile shapes that have a split-K instantiation (the ones the cost model picks for shapes with few tiles)
template <int BM, int BN, int WM, int RD, bool PERSIST, int STAGES>
constexpr bool kHasSplitK = !PERSIST && STAGES == 4 && ((BM == 128 && BN == 128) || (BM == 256 && BN == 128 && WM == 128 && RD == 2) ||
                                         (BM == 256 && BN == 256 && WM == 64 && RD == 3));

// splits > 1: every tile is computed by `splits` workgroups, split y taking K-steps y * split_steps .. and writing its
// fp32 partial tile to slice y of `partial`; the caller then runs splitk_reduce_kernel
template <int BM, int BN, int WM, int WN, int STAGES, int RD = 2, bool PERSIST = false>
hipError_t launch_variant(const GemmArgs& g0, bool out_f32, hipStream_t st, int splits = 1, int split_steps = 0, float* partial = nullptr)
{
    GemmArgs g = g0;
    g.tiles_m = (int)((g.M + BM - 1) / BM);
    g.tiles_n = (int)((g.N + BN - 1) / BN);
    if (splits > 1) {
        if constexpr (kHasSplitK<BM, BN, WM, RD, PERSIST, STAGES>) {
            constexpr int threads_s = (BM / WM) * (BN / WN) * 64;
            constexpr size_t lds_s = (size_t)STAGES * (BM + BN) / 16 * 1024 +
                                     (STAGES >= 4 ? (size_t)((BM / 16 + 1) / 2 + (BN / 16 + 1) / 2) * 1024 * (STAGES >= 6 ? 2 : 1) : (size_t)(BM + BN) / 16 * 256);
            g.out = partial;
            g.alpha = 1.0f;
            g.split_steps = split_steps;
            static LdsAttrOnce raised_s;
            auto k = gemm_mx_kernel<BM, BN, WM, WN, STAGES, true, RD, false, true>;
            hipError_t es;
            if ((es = raised_s.ensure(reinterpret_cast<const void*>(k), (int)lds_s)) != hipSuccess) return es;
            hipLaunchKernelGGL(k, dim3((unsigned)(g.tiles_m * g.tiles_n), (unsigned)splits), dim3(threads_s), lds_s, st, g);
            if ((es = hipGetLastError()) != hipSuccess) return es;
            const int64_t mn = g.M * g.N;
            const unsigned rblocks = (unsigned)std::min<int64_t>((mn + 255) / 256, 256 * 16);
            if (out_f32) hipLaunchKernelGGL(splitk_reduce_kernel<true>, dim3(rblocks), dim3(256), 0, st, partial, splits, mn, g0.alpha, g0.out);
            else hipLaunchKernelGGL(splitk_reduce_kernel<false>, dim3(rblocks), dim3(256), 0, st, partial, splits, mn, g0.alpha, g0.out);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    // operand ring + scale buffer (four and more stages: 1 KB per pair of row-blocks; three stages: 256 B per row-block)
    constexpr size_t lds = (size_t)STAGES * (BM + BN) / 16 * 1024 +
                           (STAGES >= 4 ? (size_t)((BM / 16 + 1) / 2 + (BN / 16 + 1) / 2) * 1024 * (STAGES >= 6 ? 2 : 1) : (size_t)(BM + BN) / 16 * 256);
    const int ntiles = g.tiles_m * g.tiles_n;
    int nwg = ntiles;
    if (PERSIST) {
        nwg = std::min(ntiles, compute_units() * kWgsPerCu<BM, BN, WM, WN, STAGES>);
        // the grid cap option (a testing aid: a small grid walks many tiles per workgroup)
        if (options().gemm_grid > 0) nwg = std::min(nwg, options().gemm_grid);
    }
    const dim3 grid((unsigned)nwg);
    hipError_t e;
    // the dynamic-LDS limit of a kernel is raised once per device, not on every launch
    static LdsAttrOnce raised[2];
    if (out_f32) {
        auto k = gemm_mx_kernel<BM, BN, WM, WN, STAGES, true, RD, PERSIST>;
        if ((e = raised[1].ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(threads), lds, st, g);
    } else {
        auto k = gemm_mx_kernel<BM, BN, WM, WN, STAGES, false, RD, PERSIST>;
        if ((e = raised[0].ensure(reinterpret_cast<const void*>(k), (int)lds)) != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(threads), lds, st, g);
    }
    return hipGetLastError();
}

// tile configuration by shape (the numbers of launch_gemm_mxfp4's switch)
int pick_variant_mx(int64_t M, int64_t N, int64_t K)
{
    int variant;
    if (M <= 16) variant = 4;
    else if (M <= 64) variant = 3;
    else {
        // Pick the tile by a small cost model: rounds of workgroups over the chip times (fixed cost per tile + K-steps
        // times the measured step time of that tile).  256x256 and 256x128 hold one workgroup per compute unit,
        // 128x128 two (and runs faster still when a compute unit has a single one).
        const int cus = compute_units();
        const double kt = (double)(K >> 7);
        auto tiles = [&](int bm, int bn) { return (double)((M + bm - 1) / bm) * (double)((N + bn - 1) / bn); };
        auto rounds = [](double t, double slots) { return t <= slots ? 1.0 : ceil(t / slots); };
        const double t10 = rounds(tiles(256, 256), cus) * (9.5 + kt * 0.74);
        const double t5 = rounds(tiles(256, 128), cus) * (9.0 + kt * 0.37);
        const double n2 = tiles(128, 128);
        // (0.47 us per K-step with two workgroups on a compute unit: N = 57344, K = 8192, M = 320, three rounds of 128x128 tiles
        // measured 131 us against 121 for two rounds of persistent 256x256 tiles)
        const double t2 = rounds(n2, 2.0 * cus) * (8.0 + kt * (n2 <= cus ? 0.15 : 0.47));
        variant = 10;
        double best = t10;
        if (t5 < best * 0.97) { variant = 5; best = t5; }
        if (t2 < best * 0.97) { variant = 2; best = t2; }
        // 256x192: for widths where it tiles into fewer rounds than the square tile (N = 6144 on 256 compute units:
        // 512 tiles, two full rounds of three quarters the work each, against 384 tiles = one and a half rounds)
        const double t13 = rounds(tiles(256, 192), cus) * (10.0 + kt * 0.56);
        if (t13 < best * 0.97) { variant = 13; best = t13; }
        // more 256x256 tiles than compute units: persistent workgroups, which prefetch the next tile's first stages
        // and let the output stores drain under its first K-steps (1.5-6% on such shapes, never slower)
        // -- where the tiles fill whole rounds or many of them; a ragged few rounds (N = 28672, M = 1024 / 2048: 1.75 / 3.5
        // rounds) measured 5-6 % faster with one workgroup per tile, which the hardware hands to whichever unit is free
        if (variant == 10 && tiles(256, 256) > cus) {
            const int64_t t = (int64_t)tiles(256, 256);
            if (t % cus == 0 || t >= 5 * (int64_t)cus) variant = 11;
        }
        // K around 1024: a tile is 8 K-steps, about as long as its own start-up and stores.  128x256 tiles with two
        // workgroups per compute unit overlap one workgroup's epilogue with the other's main loop: 10-13 % faster
        // there, level at K = 1536-2048, slower beyond (three stages, one and a half times the operand traffic) and
        // below (K = 512: the persistent 256x256 workgroups win).
        if ((variant == 10 || variant == 11) && K >= 768 && K <= 1280) variant = tiles(128, 256) > 2.0 * cus ? 16 : 15;
        // 128x128 tiles that leave compute units without a tile: one workgroup per unit at most, bound by what a single
        // unit can pull in -- the eight-stage ring keeps twice the bytes in flight (N = 4096, M = 128: K = 4096 14.3 ->
        // 12.5 us, K = 14336 43 -> 35 us), and eight waves of 32 x 64 (two per SIMD, one's LDS reads under the other's
        // MFMAs) are another 3-6 % faster than four of 64 x 64 (variant 17) when the unit has nothing else to run
        // (up to three quarters of the compute units busy; with more, four waves measured level or faster: N = 28672, M = 96,
        // 224 tiles: 17.4 us against 20.3)
        if (variant == 2 && n2 <= cus) variant = 4 * n2 <= 3 * cus ? 18 : 17;
    }
    return variant;
}

// Split-K plan for a product the cost model gives to 128x128, 256x128 or 256x256 tiles (more than 64 tokens).  With few
// tiles and a long K -- 65 to a few hundred tokens against a narrow layer, the batched-decoding regime -- a handful of
// compute units each stream a long K range alone and the launch is bound by the latency of their few loads in flight
// (M = 128, N = 4096, K = 14336: 32 tiles, 42 us, 0.7 TB/s).  Every tile's K range can then be cut into up to eight
// parts of at least 16 K-steps (whole scale batches of eight), each part one workgroup (17 us on that shape, reduction
// included).  The number of parts minimises an estimate in microseconds, measured on such shapes:
//     fixed cost of a tile + K-steps per part x step time + (split only) 3 for the reduction's launch
//                                                          + splits x M x N x 8 bytes of partials written and read at 4 TB/s
// and the product is split only for an estimated gain of at least 10 % (a tile of 32 K-steps is mostly fixed cost:
// N = 4096, K = 4096, M = 128 measured 14.1 us split against 13.8).  splits == 1: leave the product alone.
void plan_split_k_mx(int64_t M, int64_t N, int64_t K, int variant, int* splits, int* steps)
{
    *splits = 1;
    *steps = 0;
    int bm, bn, per_cu;
    double fixed, step_alone, step_shared;  // step time with at most one workgroup per compute unit / with more
    if (variant == 2 || variant == 17 || variant == 18) { bm = 128; bn = 128; per_cu = 2; fixed = 8.0; step_alone = variant == 2 ? 0.30 : 0.25; step_shared = 0.40; }
    else if (variant == 5) { bm = 256; bn = 128; per_cu = 1; fixed = 9.0; step_alone = step_shared = 0.45; }
    else if (variant == 10) { bm = 256; bn = 256; per_cu = 1; fixed = 9.5; step_alone = step_shared = 0.74; }
    else return;
    const int cus = compute_units();
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const int64_t slots = (int64_t)cus * per_cu;
    const int kt = (int)(K >> 7);
    const int64_t s_max = std::min<int64_t>(std::min<int64_t>(slots / tiles, kt / 16), 8);
    const double t1 = fixed + kt * (tiles <= cus ? step_alone : step_shared);
    double best = 0.9 * t1;
    for (int64_t s = 2; s <= s_max; ++s) {
        const int st = (int)(((kt + s - 1) / s + 7) / 8 * 8);
        const int64_t n = (kt + st - 1) / st;  // parts of st steps that cover K (the last may be shorter)
        if (n < 2) continue;
        const double t = fixed + st * (tiles * n <= cus ? step_alone : step_shared) + 3.0 + (double)n * (double)M * (double)N * 8.0 / 4.0e6;
        if (t < best) {
            best = t;
            *splits = (int)n;
            *steps = st;
        }
    }
}

}  // namespace

// bytes of fp32 partials a split-K run of this product needs (0: the product is not split)
size_t gemm_mx_split_k_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 64) return 0;
    int splits, steps;
    plan_split_k_mx(M, N, K, pick_variant_mx(M, N, K), &splits, &steps);
    return splits > 1 ? (size_t)splits * (size_t)M * (size_t)N * 4 : 0;
}

// variant: 0 = pick by shape; 1.. = force a tile configuration (used by the benchmark's sweep)
// partial: room for gemm_mx_split_k_bytes(M, N, K) bytes, or null (then the product is never split)
hipError_t launch_gemm_mxfp4(const void* a_codes, const void* a_scales, const void* w_codes, const void* w_scales,
                             int64_t M, int64_t N, int64_t K, void* out, bool out_f32, int variant, float alpha, void* partial,
                             hipStream_t st)
{
    GemmArgs g{};
    g.alpha = alpha;
    g.a_codes = static_cast<const uint8_t*>(a_codes);
    g.a_scales = static_cast<const uint8_t*>(a_scales);
    g.w_codes = static_cast<const uint8_t*>(w_codes);
    g.w_scales = static_cast<const uint8_t*>(w_scales);
    g.out = out;
    g.M = M;
    g.N = N;
    g.K = K;
    int splits = 1, split_steps = 0;
    if (variant == 0) {
        variant = pick_variant_mx(M, N, K);
        if (partial && M > 64) plan_split_k_mx(M, N, K, variant, &splits, &split_steps);
        if ((variant == 17 || variant == 18) && splits > 1) variant = 2;  // the parts run as four-stage workgroups, two per compute unit where needed
    }
    float* const pp = static_cast<float*>(partial);
    switch (variant) {
        case 1: return launch_variant<256, 256, 128, 128, 4>(g, out_f32, st);
        case 2: return launch_variant<128, 128, 64, 64, 4>(g, out_f32, st, splits, split_steps, pp);
        case 3: return launch_variant<64, 256, 64, 64, 4>(g, out_f32, st);
        case 4: return launch_variant<16, 256, 16, 64, 4>(g, out_f32, st);
        case 5: return launch_variant<256, 128, 128, 64, 4>(g, out_f32, st, splits, split_steps, pp);
        case 6: return launch_variant<256, 256, 128, 64, 4>(g, out_f32, st);
        case 7: return launch_variant<256, 256, 64, 128, 4>(g, out_f32, st);
        case 8: return launch_variant<256, 256, 128, 128, 4, 4>(g, out_f32, st);
        case 9: return launch_variant<256, 256, 128, 128, 4, 6>(g, out_f32, st);
        case 10: return launch_variant<256, 256, 64, 128, 4, 3>(g, out_f32, st, splits, split_steps, pp);
        case 11: return launch_variant<256, 256, 64, 128, 4, 3, true>(g, out_f32, st);
        case 12: return launch_variant<256, 128, 128, 64, 4, 2, true>(g, out_f32, st);
        case 13: return launch_variant<256, 192, 64, 96, 4, 2>(g, out_f32, st);
        case 14: return launch_variant<256, 192, 64, 96, 4, 2, true>(g, out_f32, st);
        case 15: return launch_variant<128, 256, 64, 128, 3, 3>(g, out_f32, st);
        case 16: return launch_variant<128, 256, 64, 128, 3, 3, true>(g, out_f32, st);
        case 17: return launch_variant<128, 128, 64, 64, 8>(g, out_f32, st);
        case 18: return launch_variant<128, 128, 32, 64, 8>(g, out_f32, st);
        default: return hipErrorInvalidValue;
    }
}

// compute units of the current device (asked of the runtime once per device)
int compute_units()
{
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

}  // namespace fp4mr
