// W4A8 GEMM, tiled form for more than 16 tokens: bound by the FP8 matrix cores
// when the tokens are many (prefill), a weight stream when they are few.
//
//   Y[m,n] = (sx[m] c[n]) * sum_k a[m,k] * q[k,n] * 2^e[g(k),n]   (+ T.V, LoRC)
//
// (paper Sections 1 and 3.)  A workgroup of WAVES_M x WAVES_N waves owns a
// BM x BN output tile; each wave owns WTM x WTN tiles of 16 x 16 and walks K in
// steps of 128 with v_mfma_scale_f32_16x16x128_f8f6f4 (A = E4M3 from LDS,
// B = packed E2M1 from LDS, B's E8M0 group exponent, also through LDS, in the
// instruction's scale operand -- the FP4 -> FP8 alignment is done by the
// matrix core, no unpack and no multiply).
//
// Two waves share a SIMD so that one wave's LDS reads and barrier waits hide
// behind the other's matrix instructions: two of an 8-wave workgroup that has
// the compute unit to itself (three LDS stages), or one from each of two 4-wave
// workgroups (two stages each), whose prologues, epilogues and barriers then
// fall at different times, or -- small tiles, few of them -- one from each of
// two wave groups of a workgroup that take the k-tiles in turn.  A stage
// is filled by LDS-direct loads (global_load_lds_dwordx4: every lane names a
// 16 B chunk in global memory, the wave's 64 chunks land in one contiguous
// 1 KB block of LDS), NSTAGE - 1 k-steps ahead of its use: no staging
// registers, no LDS store instructions.
// A stage keeps the activation tile as rows of 128 B with XOR-swizzled 16 B
// chunks (whole cache lines on the way in, conflict-free 16 B/lane operand
// reads on the way out); the weight tile already has its operand order in
// memory and is copied as is.
//
// The same kernel serves FP8 (E4M3) weights, the W8A8 rows of the paper's Table 2 with FP8 on both sides
// (template parameter WB = 8): a strip's k-tile is then two 1 KB halves, the first and the second four
// registers of the B operand, the operand takes two LDS reads, and the instruction is told that B is E4M3.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "zqfp_internal.h"

namespace zqfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// LDS-direct loads.  Lane l of the wave fetches 16 (or 4) bytes at gbase + voff and the hardware
// writes them to LDS byte address lds_base + 16 (4) * l; lds_base travels in M0 and is uniform.
// The compiler knows nothing of these loads or of their LDS writes: they are waited for by hand
// (wait_loads_then_barrier) and M0 has no other user in this file.
__device__ inline void lds_load16(const uint8_t* gbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(gbase) : "memory");
}
__device__ inline void lds_load4(const uint8_t* gbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_base), "v"(voff), "s"(gbase) : "memory");
}
// LDS reads issued by hand: the result registers are valid only after a wait_lds that names them
// (LDS answers a wave's requests in order; the compiler neither sees these reads nor waits for them).
template <int OFF>
__device__ inline u32x4 lds_read16(uint32_t addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF>
__device__ inline uint32_t lds_read4(uint32_t addr)
{
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// Waits until at most N of this wave's LDS reads are outstanding; the registers named are the ones
// whose use must follow the wait.
template <int N>
__device__ inline void wait_lds(u32x4& a, uint32_t& b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(u32x4& a, u32x4& b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(u32x4& a, uint32_t& b, u32x4& c, u32x4& d)
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(u32x4& a, uint32_t& b, u32x4& c)
{
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(u32x4& a, uint32_t& b, u32x4& c, u32x4& d, u32x4& e)
{
    asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e) : "n"(N));
}
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}
// Waits until at most N of this wave's loads are outstanding (loads complete in order) and for
// its LDS traffic, then joins the workgroup barrier.
template <int N>
__device__ inline void wait_loads_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// KG wave groups of WAVES_M x WAVES_N waves share the tile and take the k-tiles in turn (k-tile kt by group
// kt % KG), each with its own operands in LDS and its own accumulators; the groups' sums meet in LDS in the
// epilogue.  KG = 2 gives the small tile two waves per SIMD where the tile count leaves one workgroup per
// compute unit.  GT = threads of one group; the per-group quantities below are written in terms of it.
template <int WTM, int WTN, int WAVES_M, int WAVES_N, int NSTAGE_, int KG_ = 1, int WB = 4>
struct TileCfg {
    static_assert(WB == 4 || WB == 8, "weight bits: E2M1 or E4M3");
    static constexpr int KG = KG_;
    static constexpr int B_STRIP = 256 * WB;  // bytes of one strip (16 output channels) of one k-tile
    static constexpr int GT = 64 * WAVES_M * WAVES_N;
    static constexpr int THREADS = GT * KG;
    static constexpr int BM = WAVES_M * WTM * 16, BN = WAVES_N * WTN * 16;
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN / 16 * B_STRIP;
    static constexpr int E_BYTES = GT * 4;                    // one exponent dword per output channel (first BN used)
    static constexpr int SUB = A_BYTES + B_BYTES + E_BYTES;   // one k-tile's operands
    static constexpr int STAGE = SUB * KG;
    static constexpr int NSTAGE = NSTAGE_;
    static_assert(NSTAGE >= 2 && NSTAGE <= 8, "the loop keeps NSTAGE - 1 k-tiles in flight behind the one it multiplies");
    static constexpr int A_CHUNKS = A_BYTES / 16 / GT;  // 16 B chunks per thread
    static constexpr int B_CHUNKS = B_BYTES / 16 / GT;
    static_assert(A_BYTES % (16 * GT) == 0 && B_BYTES % (16 * GT) == 0, "tile / thread mismatch");
    static_assert(BN <= GT, "one exponent dword per thread");
    static_assert(KG == 1 || KG == 2, "one or two wave groups");
    static_assert((NSTAGE - 1) * (A_CHUNKS + B_CHUNKS + 1) <= 63, "outstanding loads must fit the 6-bit load counter");
    static_assert(NSTAGE * STAGE <= 160 * 1024, "stages exceed the LDS of a compute unit");
};

// Two waves per SIMD in every configuration (8-wave workgroups alone on a compute unit, 4-wave
// workgroups in pairs): 256 registers per lane.
template <int WTM, int WTN, int WAVES_M, int WAVES_N, int NSTAGE, int KG, bool EXACT, int WB = 4>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KG) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gemm_tile(
    const uint8_t* __restrict__ Xq, const float* __restrict__ sx, int64_t M, const uint8_t* __restrict__ blob,
    BlobLayout L, Lorc lorc, void* __restrict__ Y, int64_t ldy, int out_dtype, int tiles_m, int tiles_n, int ksplit,
    int kslice, float* __restrict__ partial)
{
    using C = TileCfg<WTM, WTN, WAVES_M, WAVES_N, NSTAGE, KG, WB>;
    static_assert(WB == 4 || WTN == 4, "E4M3 weights: three LDS reads per column block, and the counter of outstanding reads holds 15");
    constexpr int kThreads = C::THREADS;  // of the workgroup
    constexpr int kGT = C::GT;            // of one wave group
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile.  Consecutive workgroup ids go to consecutive XCDs (8 of them, one
    // L2 each), so give every XCD a contiguous range of tiles, walked in column-panels of height 8
    // so that concurrently running workgroups of an XCD share activation and weight panels in L2.
    // With a K-split every tile appears ksplit times, once per slice of kslice k-tiles.
    const int ntiles = tiles_m * tiles_n;
    int pid = blockIdx.x, slice = 0;
    {
        const int units = ntiles * ksplit;
        const int per = (units + 7) / 8;
        const int xcd = pid & 7, loc = pid >> 3;
        const int id = xcd * per + loc;
        if (id >= units) return;
        pid = id / ksplit;
        slice = id - pid * ksplit;
    }
    constexpr int GROUP_M = 8;
    const int in_group = GROUP_M * tiles_n;
    const int gid = pid / in_group;
    const int first_m = gid * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % in_group) % gsz;
    const int tn = (pid % in_group) / gsz;

    const int wg_tid = threadIdx.x, lane = wg_tid & 63;
    const int wg_wave = __builtin_amdgcn_readfirstlane(wg_tid >> 6);  // scalar: LDS block addresses go to M0
    const int kgrp = KG == 1 ? 0 : wg_wave / (kGT / 64);             // this wave's group: k-tiles kgrp, kgrp + KG, ...
    const int wave = wg_wave - kgrp * (kGT / 64), tid = wg_tid - kgrp * kGT;  // inside the group
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int col = lane & 15, lb = lane >> 4;
    const int64_t m0 = (int64_t)tm * C::BM;
    const int64_t strip0 = (int64_t)tn * (C::BN / 16);
    const int nkt_all = (int)L.nkt;                 // k-tiles of the whole K (the packed layout's stride)
    const int kt_first = slice * kslice;            // this workgroup's first k-tile
    const int nkt_wg = min(kslice, nkt_all - kt_first);  // and how many it multiplies (>= 1; a multiple of KG: the launcher's duty)
    const int kt0 = kt_first + kgrp;                // this wave group's first k-tile; its local step kt is k-tile kt0 + KG * kt
    const int nkt = nkt_wg / KG;                    // steps of every group

    // ---- load addresses: uniform base pointers plus 32-bit per-lane offsets.  Rows past M
    // and strips past the last one are clamped to the last valid one: what they produce is
    // never stored.  Load (wave, i) of the activation tile covers the 8 rows wave*8 + THREADS/8*i
    // + [0,8): lane l fetches 16 bytes of row l/8, so that 8 consecutive lanes fetch one whole 128 B
    // line, and the wave's 1 KB lands as 8 rows of 128 B.  Within a row the 16-byte chunks are
    // XOR-swizzled with the row number (slot s of row r holds chunk s ^ (r % 8)): the operand
    // reads (lane = (row, k/16 % 4), 16 B each) then spread over all LDS banks.  Load (wave, i) of
    // the weight tile is strip wave + (THREADS/64)*i, 1 KB contiguous in memory.
    const uint8_t* a_base = Xq + m0 * L.K;                    // uniform
    const uint8_t* b_base = blob + L.off_codes;               // uniform
    const uint8_t* e_base = blob + L.off_exps;                // uniform
    const int rows_here = (int)min((int64_t)C::BM, M - m0);   // >= 1
    uint32_t a_off[C::A_CHUNKS];
#pragma unroll
    for (int i = 0; i < C::A_CHUNKS; ++i) {
        const int row = (wave + (kGT / 64) * i) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ (row & 7);
        a_off[i] = (uint32_t)(min(row, rows_here - 1) * (int)L.K + 16 * chunk);
    }
    // a wave's i-th weight load is one whole strip (1 KB per k-tile): which strip is the same for all its lanes, so
    // it travels in the scalar base address and the lanes share one offset register
    const uint32_t b_lane = (uint32_t)lane * 16u;
    int64_t b_strip[C::B_CHUNKS];  // byte offset of the strip's first k-tile (wave-uniform); E4M3: of one 1 KB half of it
#pragma unroll
    for (int i = 0; i < C::B_CHUNKS; ++i) {
        const int q = wave + (kGT / 64) * i;  // 1 KB block q of the tile's weights
        const int strip = WB == 8 ? q >> 1 : q, half = WB == 8 ? q & 1 : 0;
        b_strip[i] = min(strip0 + strip, L.nstrips - 1) * nkt_all * C::B_STRIP + half * 1024;
    }
    // exponent dwords, [strip][quad][column] in memory: thread t stages the dword of column
    // t % BN of the tile; it lands in LDS as [column] and every lane later picks its own.
    const uint32_t e_off = 4u * ((uint32_t)(min(strip0 + ((tid % C::BN) >> 4), L.nstrips - 1) * L.ngq * 16) + (tid & 15));
    // LDS byte addresses (the dynamic array is the kernel's only LDS object)
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)smem + kgrp * C::SUB;  // the group's share of a stage
    const uint32_t a_dst = lds0 + wave * 1024;
    const uint32_t b_dst = lds0 + C::A_BYTES + wave * 1024;
    const uint32_t e_dst = lds0 + C::A_BYTES + C::B_BYTES + wave * 256;

    // stored exponent group of a 32-block.  Stored groups are 32 or 64 wide (then a shift of the
    // block index does it) or a multiple of 128 (then all four blocks of k-tile kt share group
    // kt / (gsb / 4), which a cursor tracks with a counter instead of dividing).  One cursor follows
    // the k-tile being computed, one the k-tile being fetched.
    struct GroupCursor { int g, sub; };
    const bool small_groups = L.gsb < 4;
    const int gq = max(1, L.gsb >> 2);
    auto group_of = [&](const GroupCursor& c, int kt, int b) {
        return small_groups ? ((kt * 4 + b) >> L.gsb_shift) : c.g;
    };
    auto advance = [&](GroupCursor& c) {  // to the group's next k-tile, KG k-tiles further on
#pragma unroll
        for (int q = 0; q < KG; ++q) {
            const int sub = c.sub + 1;
            const bool wrap = sub == gq;
            c.sub = wrap ? 0 : sub;
            c.g += wrap ? 1 : 0;
        }
    };

    // ---- one stage = NSIDE loads per wave: A_CHUNKS + B_CHUNKS 1 KB blocks and 256 B of exponents
    constexpr int NSIDE = C::A_CHUNKS + C::B_CHUNKS + 1;
    // t-th load of k-tile kt into LDS stage `stage`
    auto side_load = [&](int t, int kt, int stage, const GroupCursor& c) __attribute__((always_inline)) {
        const uint32_t st = (uint32_t)stage * C::STAGE;
        if (t < C::A_CHUNKS) lds_load16(a_base + (kt0 + KG * kt) * 128, a_off[t], st + a_dst + t * (kGT / 64) * 1024);
        else if (t < C::A_CHUNKS + C::B_CHUNKS)
            lds_load16(b_base + b_strip[t - C::A_CHUNKS] + (int64_t)(kt0 + KG * kt) * C::B_STRIP, b_lane, st + b_dst + (t - C::A_CHUNKS) * (kGT / 64) * 1024);
        else  // the dword holds 4 stored groups; the four 32-blocks of a k-tile always share one dword
            lds_load4(e_base + __builtin_amdgcn_readfirstlane((group_of(c, kt0 + KG * kt, 0) >> 2) * 64), e_off, st + e_dst);
    };

    v4f acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    // ---- operand registers.  They are refilled in place: a weight fragment and its exponent dword
    // as soon as the last matrix instruction that reads them has been issued, the activation
    // fragment almost a row block ahead of its use.  Activation fragments rotate through two
    // register sets: row block i multiplies one (fy for even i, fz for odd i) while the next
    // fragment arrives (ta, tb) and becomes the other.  In the exact mode the multiplied set holds
    // the lower exponent band and fx the upper one; the arrived fragment is split in place, one
    // dword per matrix instruction of the lower-band pass, into fx (whose old content the
    // upper-band pass has already consumed) and itself.
    u32x4 bq[WTN];        // weight fragments
    u32x4 bqh[WTN];       // E4M3 weights: their second halves
    uint32_t e_cur[WTN];  // their exponent dwords (raw until the first use in a step)
    v8i fx, fy, fz;
    u32x4 ta, tb;         // the activation fragment in flight
    GroupCursor cur_comp = {kt0 / gq, kt0 % gq}, cur_load = cur_comp;  // at this workgroup's first k-tile
    // per-lane LDS addresses inside stage 0 (the stage offset is added per step)
    const uint32_t a_addr0 = lds0 + (wm * WTM) * 2048 + col * 128 + ((lb ^ (col & 7)) * 16);
    const uint32_t a_addr1 = lds0 + (wm * WTM) * 2048 + col * 128 + ((lb ^ (col & 7) ^ 4) * 16);
    const uint32_t b_addr = lds0 + C::A_BYTES + (wn * WTN) * C::B_STRIP + lane * 16;
    const uint32_t e_addr = lds0 + C::A_BYTES + C::B_BYTES + (wn * WTN * 16 + col) * 4;
    auto as_v8i = [](const u32x4& p, const u32x4& q) {
        return (v8i){(int)p[0], (int)p[1], (int)p[2], (int)p[3], (int)q[0], (int)q[1], (int)q[2], (int)q[3]};
    };
    // The band split of the shared header in four operations instead of five: the two constants of the byte
    // selector live in registers (one scalar, one vector), so that "and" and "or" are one three-operand
    // instruction.  Plain vector operations take matrix-pipe time (about 3.5 cycles each beyond three per matrix
    // instruction, measured on register-only loops), and the split is most of them.
    constexpr bool kSplit4 = true;
    uint32_t k_sel_base = 0x03020100u, k_sel_mask = 0x04040404u;
    asm volatile("" : "+v"(k_sel_base));  // opaque: keeps the constants in registers
    asm volatile("" : "+s"(k_sel_mask));
    auto split_in_place = [&](v8i& frag, int d) __attribute__((always_inline)) {  // dword d of frag -> upper band into fx, lower band stays
        const uint32_t x = (uint32_t)frag[d];
        uint32_t h, l;
        if constexpr (kSplit4) {
            uint32_t sel;
            asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(sel) : "v"(x >> 4), "s"(k_sel_mask), "v"(k_sel_base));
            l = __builtin_amdgcn_perm(0u, x, sel);
            h = x ^ l;
        } else {
            split_exponent_bands_dword(x, h, l);
        }
        fx[d] = (int)h;
        frag[d] = (int)l;
    };
    constexpr int PASSES = EXACT ? 2 : 1;
    constexpr int RB = WB == 8 ? 3 : 2;  // LDS reads per column block: exponent dword, weight fragment (two halves if E4M3)
    static_assert(WTM % 2 == 0 && WTN >= 4 && WTN <= 8, "fragment rotation, split slots and wait schedule assume these");

    // ---- one row block of a k-step: WTN (x2 in the exact mode) matrix instructions on row block I
    // of k-tile kt, whose stage starts at LDS offset st.  In-order issue means that whatever a
    // wave puts between two matrix instructions runs in the shadow of the matrix pipe; the
    // scheduling fences pin the order written here.  LDS reads are issued and waited for by hand:
    // LDS answers in order, so "at most N reads outstanding" names exactly which have arrived.
    //   * behind the block's second instruction: the request for the next activation fragment
    //     (row block I + 1, or row block 0 of the next stage st_next when I is the last and NEXT);
    //   * last block only (it runs behind the step's barrier, see below): one per instruction, the
    //     requests for k-tile kt + NSTAGE into this step's stage (LOAD) and, behind the last instruction
    //     that reads them, the next step's weight fragments and exponent dwords (NEXT);
    //   * block 0: instruction j waits for its own fragment j only (read_b order: e0 b0 e1 b1 ...; E4M3
    //     weights: e0 b0 b0' e1 ...): RB (WTN - 1 - j) younger reads, RB = 2 or 3 per column block, plus the
    //     2 of the activation request once that is out.
    auto row_block = [&](auto i_tag, int kt, uint32_t st, uint32_t st_next, int stage, auto load_tag, auto next_tag) __attribute__((always_inline)) {
        constexpr int I = decltype(i_tag)::value;
        constexpr bool LOAD = decltype(load_tag)::value;
        constexpr bool NEXT = decltype(next_tag)::value;
        constexpr bool last_block = I == WTM - 1;
        constexpr bool fetch = !last_block || NEXT;
        v8i& cur = (I & 1) ? fz : fy;
        v8i& inc = (I & 1) ? fy : fz;
        const int esh = 8 * (group_of(cur_comp, kt0 + KG * kt, lb) & 3);  // this lane's exponent byte: (stored group & 3) of the dword
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, PASSES>([&](auto p_tag) __attribute__((always_inline)) {
            constexpr int P = decltype(p_tag)::value;
            static_for<0, WTN>([&](auto j_tag) __attribute__((always_inline)) {
                constexpr int J = decltype(j_tag)::value;
                if constexpr (I == 0 && P == 0) {
                    constexpr int YOUNGER = RB * (WTN - 1 - J) + (J >= 2 ? 2 : 0);
                    if constexpr (J == 0 && !EXACT) {  // the fragment that arrived during the previous block
                        if constexpr (WB == 8) wait_lds<YOUNGER>(bq[J], e_cur[J], bqh[J], ta, tb);
                        else wait_lds<YOUNGER>(bq[J], e_cur[J], ta, tb);
                        cur = as_v8i(ta, tb);
                    } else {
                        if constexpr (WB == 8) wait_lds<YOUNGER>(bq[J], e_cur[J], bqh[J]);
                        else wait_lds<YOUNGER>(bq[J], e_cur[J]);
                    }
                    e_cur[J] >>= esh;
                } else if constexpr (I > 0 && P == 0 && J == 0 && !EXACT) {
                    wait_lds<0>(ta, tb);
                    cur = as_v8i(ta, tb);
                }
                if constexpr (EXACT && P == 1 && J == 0 && fetch) {
                    wait_lds<0>(ta, tb);
                    inc = as_v8i(ta, tb);
                }
                const v8i& op = (EXACT && P == 0) ? fx : cur;
                // cbsz 0: A is E4M3; blgp 4: B is E2M1 (blgp 0: E4M3); A scale byte 127 = 2^0; B scale = group exponent
                if constexpr (WB == 8) {
                    const v8i bv = {(int)bq[J][0], (int)bq[J][1], (int)bq[J][2], (int)bq[J][3], (int)bqh[J][0], (int)bqh[J][1], (int)bqh[J][2], (int)bqh[J][3]};
                    acc[I][J] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(op, bv, acc[I][J], 0, 0, 0, 127, 0, (int)e_cur[J]);
                } else {
                    const v8i bv = {(int)bq[J][0], (int)bq[J][1], (int)bq[J][2], (int)bq[J][3], 0, 0, 0, 0};
                    acc[I][J] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(op, bv, acc[I][J], 0, 4, 0, 127, 0, (int)e_cur[J]);
                }
                if constexpr (P == 0 && J == 1 && fetch) {
                    if constexpr (!last_block) {
                        ta = lds_read16<(I + 1) * 2048>(a_addr0 + st);
                        tb = lds_read16<(I + 1) * 2048>(a_addr1 + st);
                    } else {
                        ta = lds_read16<0>(a_addr0 + st_next);
                        tb = lds_read16<0>(a_addr1 + st_next);
                    }
                }
                if constexpr (EXACT && P == 1 && fetch) {
#pragma unroll
                    for (int d = J * 8 / WTN; d < (J + 1) * 8 / WTN; ++d) split_in_place(inc, d);
                }
                if constexpr (last_block) {
                    constexpr int T = P * WTN + J;  // position in the block's matrix-instruction stream
                    constexpr int PER = (NSIDE + WTN * PASSES - 1) / (WTN * PASSES);  // loads per slot
#pragma unroll
                    for (int q = 0; q < PER; ++q)
                        if (LOAD && T * PER + q < NSIDE) side_load(T * PER + q, kt + NSTAGE, stage, cur_load);
                    if constexpr (NEXT && P == PASSES - 1) {
                        e_cur[J] = lds_read4<J * 64>(e_addr + st_next);
                        bq[J] = lds_read16<J * C::B_STRIP>(b_addr + st_next);
                        if constexpr (WB == 8) bqh[J] = lds_read16<J * C::B_STRIP + 1024>(b_addr + st_next);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    auto stage_off = [](int stage) { return (uint32_t)stage * C::STAGE; };
    auto next = [](int st) { return st == C::NSTAGE - 1 ? 0 : st + 1; };
    // row blocks 0 .. WTM - 2 of step kt, then the step's barrier.  It sits BEFORE the last row
    // block: by then every read of this stage has been issued (the last activation fragment is
    // requested one block ahead), so behind the barrier the stage is free for k-tile kt + NSTAGE, and
    // the next stage is complete: each wave has waited for all of its loads but the WAIT that may
    // belong to k-tile kt + 2.
    auto head_blocks = [&](int kt, int stage, auto wait_tag) __attribute__((always_inline)) {
        const uint32_t st = stage_off(stage);
        static_for<0, WTM - 1>([&](auto i_tag) __attribute__((always_inline)) { row_block(i_tag, kt, st, 0u, stage, no{}, no{}); });
        wait_loads_then_barrier<decltype(wait_tag)::value>();
    };

    // ---- prologue: k-tiles 0 .. NSTAGE - 1 (as far as they exist) into stages of the same number; the
    // first operands into registers.  The fetch cursor ends at k-tile NSTAGE when more will be requested.
    static_for<0, NSTAGE>([&](auto t_tag) __attribute__((always_inline)) {
        constexpr int TILE = decltype(t_tag)::value;
        if (TILE < nkt) {
            if constexpr (TILE > 0) advance(cur_load);
#pragma unroll
            for (int t = 0; t < NSIDE; ++t) side_load(t, TILE, TILE, cur_load);
        }
    });
    if (nkt >= NSTAGE) advance(cur_load);
    // k-tile 0 has landed, for every wave, once all but the later tiles' loads are done.  A pipeline shorter than
    // the stages waits for everything here, so that the first step's barrier below needs no second form: the code
    // behind this point has LDS reads in flight, and a branch with two copies of it invites the register
    // allocator to copy a fragment register between its read and its wait (the build checks the listing for that).
    if (nkt >= NSTAGE) wait_loads_then_barrier<(NSTAGE - 1) * NSIDE>();
    else wait_loads_then_barrier<0>();
    ta = lds_read16<0>(a_addr0);
    tb = lds_read16<0>(a_addr1);
    static_for<0, WTN>([&](auto j_tag) __attribute__((always_inline)) {
        constexpr int J = decltype(j_tag)::value;
        e_cur[J] = lds_read4<J * 64>(e_addr);
        bq[J] = lds_read16<J * C::B_STRIP>(b_addr);
        if constexpr (WB == 8) bqh[J] = lds_read16<J * C::B_STRIP + 1024>(b_addr);
    });
    if constexpr (EXACT) {  // the fast mode picks ta, tb up at its first matrix instruction
        wait_lds<(RB * WTN < 15 ? RB * WTN : 15)>(ta, tb);  // the counter holds 15 at most
        fy = as_v8i(ta, tb);
#pragma unroll
        for (int d = 0; d < 8; ++d) split_in_place(fy, d);
    }

    // ---- main loop.  Step kt computes stage kt % NSTAGE; the k-tiles behind it (kt + 1 .. kt + NSTAGE - 1)
    // are in the other stages or on their way, k-tile kt + NSTAGE is requested into
    // stage kt % NSTAGE behind the step's barrier: NSTAGE - 1 steps of slack for the memory latency
    // (most of one with two stages, where two workgroups share a compute unit and fill each other's
    // gaps; five with the six stages of the small tile, whose lone workgroup is a weight stream).  The loop is rotated so that no LDS read is in flight across its back edge: an iteration is
    // the last row block of step kt followed by the first blocks of step kt + 1 and that step's barrier,
    // at which the loads of k-tile kt + 2 must have landed and only younger ones (those of k-tiles
    // kt + 3 .. kt + NSTAGE) may be outstanding.  The last steps request nothing and are peeled.
    using W1 = std::integral_constant<int, (NSTAGE - 2) * NSIDE>;
    using W0 = std::integral_constant<int, 0>;
    int stage = 0;
    head_blocks(0, 0, W1{});  // k-tiles 2 .. NSTAGE - 1 may still be on their way (a shorter pipeline has nothing outstanding)
    int kt = 0;
    for (; kt + NSTAGE < nkt; ++kt) {  // k-tile kt + NSTAGE exists
        row_block(std::integral_constant<int, WTM - 1>{}, kt, stage_off(stage), stage_off(next(stage)), stage, yes{}, yes{});
        advance(cur_comp);
        advance(cur_load);
        stage = next(stage);
        head_blocks(kt + 1, stage, W1{});
    }
    for (; kt + 1 < nkt; ++kt) {  // nothing left to request: at the barrier no load may be outstanding
        row_block(std::integral_constant<int, WTM - 1>{}, kt, stage_off(stage), stage_off(next(stage)), stage, no{}, yes{});
        advance(cur_comp);
        stage = next(stage);
        head_blocks(kt + 1, stage, W0{});
    }
    row_block(std::integral_constant<int, WTM - 1>{}, kt, stage_off(stage), 0u, stage, no{}, no{});

    // ---- epilogue.  D[row][col] of a 16x16 tile sits in lane 16*(row/4)+col, register row%4:
    // good for the scale / LoRC arithmetic (one column per lane), bad for stores (64 B runs).
    // Each wave therefore passes its 16 x (16*WTN) slabs through a private LDS patch (row stride
    // 16*WTN + 4 floats: the four row groups of a store land on disjoint banks, rows stay 16 B
    // aligned) and writes them out as 16 B per lane, whole rows of the slab at a time.
    constexpr int SLAB_N = 16 * WTN, SLAB_LD = SLAB_N + 4;
    static_assert(C::THREADS / 64 * 16 * SLAB_LD * 4 <= C::NSTAGE * C::STAGE, "epilogue patch does not fit the stages");
    __syncthreads();  // every wave is done reading the stages
    if constexpr (KG == 2) {  // the second wave group hands its sums over: acc = group 0 + group 1, a fixed order
        static_assert(WTM * WTN * kGT * 16 <= C::NSTAGE * C::STAGE, "hand-over area does not fit the stages");
        v4f* comb = reinterpret_cast<v4f*>(smem);
        if (kgrp == 1) {
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j) comb[(i * WTN + j) * kGT + tid] = acc[i][j];
        }
        __syncthreads();
        if (kgrp == 0) {
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j) acc[i][j] += comb[(i * WTN + j) * kGT + tid];
        }
        __syncthreads();  // the area is reused below
    }
    float* patch = reinterpret_cast<float*>(smem) + wave * (16 * SLAB_LD);
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);
    const int64_t n_wave = (strip0 + wn * WTN) * 16;
    // With a K-split the workgroup hands its raw float32 sums to slice `slice` of the workspace
    // ([ksplit][M][Np]); scales and LoRC are applied by the kernel that adds the slices up.
    const bool raw = ksplit > 1;
    if (raw) {
        Y = partial + (int64_t)slice * M * L.Np;
        ldy = L.Np;
        out_dtype = 0;
    }
    float cn[WTN];
#pragma unroll
    for (int j = 0; j < WTN; ++j) cn[j] = raw ? 1.0f : colscale[min(n_wave + j * 16 + col, L.Np - 1)];
    // LoRC of rank <= 8 (the paper's setting): the tile's rows of T and columns of V go through LDS
    // once (zero-padded to rank 8, V converted to binary32), so that the 8 fused multiply-adds per
    // output read registers filled by two 16-byte LDS reads per row and per column.
    constexpr int RL = 8;
    constexpr int PATCH_BYTES = C::THREADS / 64 * 16 * SLAB_LD * 4;
    static_assert(PATCH_BYTES + (C::BM + C::BN) * RL * 4 <= C::NSTAGE * C::STAGE, "LoRC tiles do not fit the stages");
    float* Ts = reinterpret_cast<float*>(smem + PATCH_BYTES);  // [BM][RL]
    float* Vs = Ts + C::BM * RL;                               // [BN][RL]
    const int rk = raw ? 0 : lorc.r;
    const bool lorc_lds = rk > 0 && rk <= RL;
    if (lorc_lds) {
        for (int idx = wg_tid; idx < C::BM * RL; idx += kThreads) {
            const int row = idx / RL, q = idx % RL;
            Ts[idx] = q < rk ? lorc.T[min(m0 + row, M - 1) * rk + q] : 0.f;
        }
        for (int idx = wg_tid; idx < RL * C::BN; idx += kThreads) {
            const int q = idx / C::BN, c = idx % C::BN;
            const int64_t n = min(strip0 * 16 + c, L.N - 1);
            Vs[c * RL + q] = q < rk ? half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]) : 0.f;
        }
        __syncthreads();
    }
    if (KG == 2 && kgrp != 0) return;  // no barrier below: the first group alone writes the tile out
    constexpr int LPR = SLAB_N / 4;   // lanes per slab row when each lane carries 4 columns
    constexpr int RPI = 64 / LPR;     // slab rows per store instruction (lanes beyond RPI * LPR idle when 64 % LPR != 0)
    static_assert(RPI >= 1 && 16 % RPI == 0, "slab rows per store instruction");
    const int srow = lane / LPR, scol = (lane % LPR) * 4;
    const bool lane_stores = lane < RPI * LPR;
    const bool vec_ok = (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
#pragma unroll
    for (int i = 0; i < WTM; ++i) {
        const int64_t m_slab = m0 + (wm * WTM + i) * 16;
        float sxm[4];
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) sxm[rg] = raw ? 1.0f : sx[min(m_slab + 4 * lb + rg, M - 1)];
        v4f tl[4][RL / 4];
        if (lorc_lds) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg)
#pragma unroll
                for (int h = 0; h < RL / 4; ++h)
                    tl[rg][h] = *reinterpret_cast<const v4f*>(Ts + ((wm * WTM + i) * 16 + 4 * lb + rg) * RL + 4 * h);
        }
#pragma unroll
        for (int j = 0; j < WTN; ++j) {
            const int64_t n = min(n_wave + j * 16 + col, L.N - 1);
            v4f vl[RL / 4];
            if (lorc_lds) {
#pragma unroll
                for (int h = 0; h < RL / 4; ++h)
                    vl[h] = *reinterpret_cast<const v4f*>(Vs + ((wn * WTN + j) * 16 + col) * RL + 4 * h);
            }
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float y = (sxm[rg] * cn[j]) * acc[i][j][rg];
                if (lorc_lds) {
#pragma unroll
                    for (int q = 0; q < RL; ++q) y = fmaf(tl[rg][q / 4][q % 4], vl[q / 4][q % 4], y);  // padding adds 0 * 0
                } else if (rk > 0) {  // larger ranks: read in place
                    const float* t = lorc.T + min(m_slab + 4 * lb + rg, M - 1) * rk;
                    for (int q = 0; q < rk; ++q) y = fmaf(t[q], half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]), y);
                }
                patch[(4 * lb + rg) * SLAB_LD + j * 16 + col] = y;
            }
        }
#pragma unroll
        for (int t = 0; t < 16 / RPI; ++t) {
            const int r = lane_stores ? t * RPI + srow : 0;
            const v4f y = *reinterpret_cast<const v4f*>(patch + r * SLAB_LD + scol);
            const int64_t m = m_slab + r, n = n_wave + scol;
            if (!lane_stores || m >= M || n >= L.N) continue;
            if (out_dtype == 0) {
                float* dst = reinterpret_cast<float*>(Y) + m * ldy + n;
                if (vec_ok && n + 3 < L.N) {
                    *reinterpret_cast<v4f*>(dst) = y;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (n + q < L.N) dst[q] = y[q];
                }
            } else {
                uint16_t* dst = reinterpret_cast<uint16_t*>(Y) + m * ldy + n;
                if (vec_ok && n + 3 < L.N) {
                    uint2 pk;
                    pk.x = (uint32_t)f32_to_bf16_bits(y[0]) | ((uint32_t)f32_to_bf16_bits(y[1]) << 16);
                    pk.y = (uint32_t)f32_to_bf16_bits(y[2]) | ((uint32_t)f32_to_bf16_bits(y[3]) << 16);
                    *reinterpret_cast<uint2*>(dst) = pk;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (n + q < L.N) dst[q] = f32_to_bf16_bits(y[q]);
                }
            }
        }
    }
}

// Sums the K slices of a split launch in slice order and applies what the tile epilogue would have:
// Y[m,n] = (sx[m] c[n]) * sum_s partial[s][m][n] (+ T.V).  Four consecutive columns per thread.
__global__ __launch_bounds__(256) void k_splitk_reduce(const float* __restrict__ partial, int ksplit, int64_t M,
                                                     const uint8_t* __restrict__ blob, BlobLayout L,
                                                     const float* __restrict__ sx, Lorc lorc, void* __restrict__ Y,
                                                     int64_t ldy, int out_dtype)
{
    const int64_t quads = L.Np / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * quads) return;
    const int64_t m = idx / quads, n0 = (idx - m * quads) * 4;
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < ksplit; ++s) acc += *reinterpret_cast<const v4f*>(partial + ((int64_t)s * M + m) * L.Np + n0);
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);
    const float sm = sx[m];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t n = n0 + q;
        if (n >= L.N) break;
        float y = (sm * colscale[n]) * acc[q];
        for (int j = 0; j < lorc.r; ++j) y = fmaf(lorc.T[m * lorc.r + j], half_bits_to_f32(lorc.V[(int64_t)j * L.N + n]), y);
        if (out_dtype == 0) reinterpret_cast<float*>(Y)[m * ldy + n] = y;
        else reinterpret_cast<uint16_t*>(Y)[m * ldy + n] = f32_to_bf16_bits(y);
    }
}


template <int WTM, int WTN, int WAVES_M, int WAVES_N, int NSTAGE, int KG, bool EXACT, int WB = 4>
hipError_t launch_cfg(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L, Lorc lorc,
                      void* Y, int64_t ldy, int out_dtype, int ksplit, int kslice, float* partial, hipStream_t s)
{
    using C = TileCfg<WTM, WTN, WAVES_M, WAVES_N, NSTAGE, KG, WB>;
    const int tiles_m = (int)((M + C::BM - 1) / C::BM), tiles_n = (int)((L.Np + C::BN - 1) / C::BN);
    const int units = tiles_m * tiles_n * ksplit;
    const int per = (units + 7) / 8;
    const size_t smem = C::NSTAGE * C::STAGE;
    auto kern = k_gemm_tile<WTM, WTN, WAVES_M, WAVES_N, NSTAGE, KG, EXACT, WB>;
    static OnceStatus attr;  // raising the dynamic LDS limit is a per-function, per-process setting (one flag per instantiation)
    if (hipError_t e = run_once(attr, [&] {
            return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        }); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(C::THREADS), smem, s, Xq, sx, M, blob, L, lorc, Y, ldy,
                       out_dtype, tiles_m, tiles_n, ksplit, kslice, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || ksplit == 1) return e;
    return launch_splitk_reduce(partial, ksplit, M, blob, L, sx, lorc, Y, ldy, out_dtype, s);
}

template <bool EXACT>
hipError_t launch_pick(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L, Lorc lorc,
                       void* Y, int64_t ldy, int out_dtype, void* workspace, hipStream_t s)
{
    TilePlan p = effective_tile_plan(M, L.Np, L.nkt);
    if (workspace == nullptr) { p.ksplit = 1; p.kslice = (int)L.nkt; }  // no room for partial tiles: one slice
    float* ws = static_cast<float*>(workspace);
#define ZQ_TILE(WTM, WTN, WM, WN, NST, KG) \
    return launch_cfg<WTM, WTN, WM, WN, NST, KG, EXACT>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, p.ksplit, p.kslice, ws, s)
    if (p.bm == 256) ZQ_TILE(4, 8, 4, 2, 3, 1);
    if (p.bm == 128 && p.bn == 256) ZQ_TILE(4, 8, 2, 2, 2, 1);
    if (p.bm == 128 && p.bn == 192) ZQ_TILE(4, 6, 2, 2, 2, 1);
    if (p.bm == 128) ZQ_TILE(4, 4, 2, 2, 3, 1);
    // 64-row tiles.  Two wave groups need an even number of k-tiles in every slice.
    if (p.ksplit >= 2 && !p.forced) {  // half as many slices (of even length), two wave groups each: half the partial tiles to add up
        const int64_t tiles = ((M + 63) / 64) * ((L.Np + 127) / 128);
        const int want = (p.ksplit + 1) / 2;
        int kslice = (int)((L.nkt + want - 1) / want);
        kslice += kslice & 1;
        const int ksplit = (int)((L.nkt + kslice - 1) / kslice);
        const int tail = (int)L.nkt - (ksplit - 1) * kslice;
        if (tiles * ksplit <= 256 && tail > 0 && tail % 2 == 0) { p.ksplit = ksplit; p.kslice = kslice; p.kg = 2; }
    }
    const bool even_slices = p.kslice % 2 == 0 && ((int)L.nkt - (p.ksplit - 1) * p.kslice) % 2 == 0;
    const bool two_groups = p.kg == 2 && even_slices;
    if (p.bn == 256) { if (two_groups) ZQ_TILE(2, 8, 2, 2, 3, 2); ZQ_TILE(2, 8, 2, 2, 3, 1); }
    if (p.bn == 192) { if (two_groups) ZQ_TILE(2, 6, 2, 2, 3, 2); ZQ_TILE(2, 6, 2, 2, 3, 1); }
    if (two_groups) ZQ_TILE(2, 4, 2, 2, 3, 2);
    ZQ_TILE(2, 4, 2, 2, 3, 1);
#undef ZQ_TILE
}

// E4M3 weights: 128 x 128 tiles, two workgroups per compute unit, once there is more than one of them per compute
// unit; below that 64 x 128 tiles, with two wave groups while at most one workgroup per compute unit is left (and
// the k-tiles can be dealt out in pairs).  No K-split: the W8A8 entry point takes no workspace.
template <bool EXACT>
hipError_t launch_pick_w8(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L, Lorc lorc,
                          void* Y, int64_t ldy, int out_dtype, hipStream_t s)
{
    auto tiles = [&](int bm) { return ((M + bm - 1) / bm) * ((L.Np + 127) / 128); };
    int bm = tiles(128) > 256 ? 128 : 64;
    int kg = bm == 64 && tiles(64) <= 256 ? 2 : 1;
    const TilePlan f = effective_tile_plan(M, L.Np, L.nkt);
    if (f.forced && f.bn == 128 && (f.bm == 64 || f.bm == 128)) { bm = f.bm; kg = f.bm == 64 ? f.kg : 1; }
    if (L.nkt & 1) kg = 1;
#define ZQ_TILE8(WTM, NST, KG) \
    return launch_cfg<WTM, 4, 2, 2, NST, KG, EXACT, 8>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, 1, (int)L.nkt, nullptr, s)
    if (bm == 128) ZQ_TILE8(4, 2, 1);
    if (kg == 2) ZQ_TILE8(2, 3, 2);
    ZQ_TILE8(2, 3, 1);
#undef ZQ_TILE8
}

std::atomic<uint32_t> g_forced_plan{0};  // bm | bn << 10 | ksplit << 20 | kg << 28; 0 = automatic

}  // namespace

hipError_t launch_splitk_reduce(const float* partial, int slices, int64_t M, const uint8_t* blob, const BlobLayout& L,
                                const float* sx, Lorc lorc, void* Y, int64_t ldy, int out_dtype, hipStream_t s)
{
    const int64_t threads = M * (L.Np / 4);
    hipLaunchKernelGGL(k_splitk_reduce, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, partial, slices, M, blob, L,
                       sx, lorc, Y, ldy, out_dtype);
    return hipGetLastError();
}

bool gemm_tile_supported(int64_t M, const BlobLayout& L) { return M > 16 && L.N >= 64; }

// ---- planning.  Measured on LLaMA-7B / 13B / 70B and OPT shapes (exact accumulation), the time of a launch is
// close to  3 + t * (e + s * k-tiles)  microseconds, t = the most tiles any compute unit gets: e is a tile's
// prologue and epilogue, s its k-step.  Small tiles cost more per output (plain vector work per matrix
// instruction grows as a wave's tile narrows, and it takes matrix-pipe time), large tiles come in coarser
// rounds.  A compute unit that holds a single four-wave workgroup has one wave per SIMD and nothing to fill
// its stalls with: 1.3 times slower.  The planner takes the cheapest.
struct TileKind {
    int bm, bn, kg;
    float e, s;
};
constexpr TileKind kTileKinds[] = {
    // least-squares fit (relative error) to 527 timings: seven weight shapes with 16 ... 224 k-tiles, 64 ... 4096 tokens
    {64, 128, 2, 3.8f, 0.368f},   // two wave groups: one workgroup per compute unit, so at most 256 tiles
    {64, 192, 2, 6.0f, 0.477f},
    {64, 256, 2, 6.8f, 0.584f},
    {64, 128, 1, 2.1f, 0.368f},
    {64, 192, 1, 3.3f, 0.464f},
    {64, 256, 1, 4.5f, 0.549f},
    {128, 128, 1, 4.3f, 0.632f},
    {128, 192, 1, 6.6f, 0.778f},
    {128, 256, 1, 8.6f, 0.928f},
    {256, 256, 1, 12.4f, 2.009f},
};

TilePlan plan_tiles(int64_t M, int64_t Np, int64_t nkt)
{
    constexpr int64_t kCUs = 256;  // MI355X
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((Np + bn - 1) / bn); };
    TilePlan p{64, 128, 1, 1, (int)nkt};
    // Few output tiles, long K (down-projections at small M): even 64 x 128 tiles fill less than a third of the
    // chip, so K is cut into slices of at least 8 k-steps.
    {
        const int64_t slots = 2 * kCUs, nt = tiles(64, 128);
        int64_t want = slots / nt;
        if (want > 16) want = 16;
        if (want > nkt / 8) want = nkt / 8;
        if (want >= 3) {
            // The slices' trip through memory must pay for itself: against the un-split launch (two wave groups, at
            // most one tile per compute unit here) the split saves K-steps and costs a second kernel and the
            // partial sums written, read back and summed.  The launch will halve the slice count where two wave
            // groups can take the halves (launch_pick), which is what is priced.  Measured on K = N = 4096: splitting
            // wins up to 128 tokens (17.0 against 18.1 us) and loses from 192 on (21.1 against 18.4 at 256), while
            // K = 11008 gains at every token count that gets here (256 tokens: 29.6 against 38.1 us).
            const int kslice = (int)((nkt + want - 1) / want), ksplit = (int)((nkt + kslice - 1) / kslice);
            const float eff = (float)((ksplit + 1) / 2);
            const float trip_us = (2.0f * eff + 1.0f) * (float)M * (float)Np * 4.0f / 2.5e6f;  // measured: 2.5 TB/s, second launch included
            const float split_us = 3.8f + 0.368f * (float)nkt / eff + trip_us, unsplit_us = 3.8f + 0.368f * (float)nkt;
            if (split_us < unsplit_us) {
                p.kslice = kslice;
                p.ksplit = ksplit;
                return p;
            }
        }
    }
    // Many rounds of large tiles: 128 x 256, two workgroups per compute unit that fill each other's gaps.
    const int64_t n256 = tiles(256, 256);
    if (n256 >= kCUs * 3 / 2) { p.bm = 128; p.bn = 256; return p; }
    float best = 0.f;
    bool have = false;
    for (const TileKind& k : kTileKinds) {
        const int64_t t = tiles(k.bm, k.bn);
        if (k.kg == 2 && (t > kCUs || (nkt & 1))) continue;
        if (k.bm > 64 && M <= 64) continue;
        const float per_cu = (float)((t + kCUs - 1) / kCUs);
        const bool lone_waves = t <= kCUs && k.kg == 1 && k.bm < 256;
        const float cost = 3.0f + per_cu * (k.e + k.s * (float)nkt) * (lone_waves ? 1.3f : 1.0f);
        if (!have || cost < best) { best = cost; have = true; p.bm = k.bm; p.bn = k.bn; p.kg = k.kg; }
    }
    return p;
}

bool force_tile_plan(int bm, int bn, int ksplit, int kg)
{
    if (bm == 0 && bn == 0 && ksplit == 0) { g_forced_plan.store(0); return true; }
    const bool shape_ok = (bm == 64 && (bn == 128 || bn == 192 || bn == 256)) ||
                          (bm == 128 && (bn == 128 || bn == 192 || bn == 256)) || (bm == 256 && bn == 256);
    if (!shape_ok || ksplit < 1 || ksplit > 64 || kg < 1 || kg > 2 || (kg == 2 && bm != 64)) return false;
    g_forced_plan.store((uint32_t)bm | ((uint32_t)bn << 10) | ((uint32_t)ksplit << 20) | ((uint32_t)kg << 28));
    return true;
}

TilePlan effective_tile_plan(int64_t M, int64_t Np, int64_t nkt)
{
    const uint32_t f = g_forced_plan.load(std::memory_order_relaxed);
    if (f == 0) return plan_tiles(M, Np, nkt);
    TilePlan p;
    p.bm = (int)(f & 1023u); p.bn = (int)((f >> 10) & 1023u);
    p.kg = (int)(f >> 28);
    const int want = (int)std::min<int64_t>((int64_t)((f >> 20) & 255u), nkt);
    p.kslice = (int)((nkt + want - 1) / want);
    p.ksplit = (int)((nkt + p.kslice - 1) / p.kslice);
    p.forced = true;
    return p;
}

hipError_t launch_gemm_w8_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                               Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, hipStream_t s)
{
    if (M == 0 || L.N == 0) return hipSuccess;
    return accum == 0 ? launch_pick_w8<true>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s)
                      : launch_pick_w8<false>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
}

hipError_t launch_gemm_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                            Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, void* workspace, hipStream_t s)
{
    return accum == 0 ? launch_pick<true>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, workspace, s)
                      : launch_pick<false>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, workspace, s);
}

}  // namespace zqfp
