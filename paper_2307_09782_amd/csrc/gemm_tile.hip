// W4A8 GEMM, tiled form for many tokens (prefill): bound by the FP8 matrix
// cores.
//
//   Y[m,n] = (sx[m] c[n]) * sum_k a[m,k] * q[k,n] * 2^e[g(k),n]   (+ T.V, LoRC)
//
// (paper Sections 1 and 3.)  A workgroup of WAVES_M x WAVES_N waves owns a
// BM x BN output tile; each wave owns WTM x WTN tiles of 16 x 16 and walks K in
// steps of 128 with v_mfma_scale_f32_16x16x128_f8f6f4 (A = E4M3 from LDS,
// B = packed E2M1 from LDS, B's E8M0 group exponent straight from global
// memory into the instruction's scale operand -- the FP4 -> FP8 alignment is
// done by the matrix core, no unpack and no multiply).
//
// Two waves share a SIMD so that one wave's LDS reads and barrier waits hide
// behind the other's matrix instructions.  LDS holds three stages.  A stage
// is filled by LDS-direct loads (global_load_lds_dwordx4: every lane names a
// 16 B chunk in global memory, the wave's 64 chunks land in one contiguous
// 1 KB block of LDS), two k-steps ahead of its use: no staging registers, no
// LDS store instructions, and two k-steps of slack for the memory latency.
// A stage keeps the activation tile as rows of 128 B with XOR-swizzled 16 B
// chunks (whole cache lines on the way in, conflict-free 16 B/lane operand
// reads on the way out); the weight tile already has its operand order in
// memory and is copied as is.
#include <type_traits>

#include "zqfp_internal.h"

namespace zqfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

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
// Waits until at most N of this wave's loads are outstanding (loads complete in order) and for
// its LDS traffic, then joins the workgroup barrier.
template <int N>
__device__ inline void wait_loads_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int WTM, int WTN, int WAVES_M, int WAVES_N>
struct TileCfg {
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int BM = WAVES_M * WTM * 16, BN = WAVES_N * WTN * 16;
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 64;
    static constexpr int E_BYTES = THREADS * 4;               // one exponent dword per output channel (first BN used)
    static constexpr int STAGE = A_BYTES + B_BYTES + E_BYTES;
    static constexpr int NSTAGE = 3;
    static constexpr int A_CHUNKS = A_BYTES / 16 / THREADS;  // 16 B chunks per thread
    static constexpr int B_CHUNKS = B_BYTES / 16 / THREADS;
    static_assert(A_BYTES % (16 * THREADS) == 0 && B_BYTES % (16 * THREADS) == 0, "tile / thread mismatch");
    static_assert(BN <= THREADS, "one exponent dword per thread");
};

// Two waves per SIMD in every configuration (8-wave workgroups alone on a compute unit, 4-wave
// workgroups in pairs): 256 registers per lane.
template <int WTM, int WTN, int WAVES_M, int WAVES_N, bool EXACT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gemm_tile(
    const uint8_t* __restrict__ Xq, const float* __restrict__ sx, int64_t M, const uint8_t* __restrict__ blob,
    BlobLayout L, Lorc lorc, void* __restrict__ Y, int64_t ldy, int out_dtype, int tiles_m, int tiles_n)
{
    using C = TileCfg<WTM, WTN, WAVES_M, WAVES_N>;
    constexpr int kThreads = C::THREADS;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile.  Consecutive workgroup ids go to consecutive XCDs (8 of them, one
    // L2 each), so give every XCD a contiguous range of tiles, walked in column-panels of height 8
    // so that concurrently running workgroups of an XCD share activation and weight panels in L2.
    const int ntiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int per = (ntiles + 7) / 8;
        const int xcd = pid & 7, loc = pid >> 3;
        const int id = xcd * per + loc;
        if (id >= ntiles) return;
        pid = id;
    }
    constexpr int GROUP_M = 8;
    const int in_group = GROUP_M * tiles_n;
    const int gid = pid / in_group;
    const int first_m = gid * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % in_group) % gsz;
    const int tn = (pid % in_group) / gsz;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: LDS block addresses go to M0
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int col = lane & 15, lb = lane >> 4;
    const int64_t m0 = (int64_t)tm * C::BM;
    const int64_t strip0 = (int64_t)tn * (C::BN / 16);
    const int nkt = (int)L.nkt;

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
    uint32_t a_off[C::A_CHUNKS], b_off[C::B_CHUNKS];
#pragma unroll
    for (int i = 0; i < C::A_CHUNKS; ++i) {
        const int row = (wave + (kThreads / 64) * i) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ (row & 7);
        a_off[i] = (uint32_t)(min(row, rows_here - 1) * (int)L.K + 16 * chunk);
    }
#pragma unroll
    for (int i = 0; i < C::B_CHUNKS; ++i) {
        const int cidx = tid + kThreads * i;
        const int64_t strip = min(strip0 + (cidx >> 6), L.nstrips - 1);
        b_off[i] = (uint32_t)((strip * nkt * 64 + (cidx & 63)) * 16);
    }
    // exponent dwords, [strip][quad][column] in memory: thread t stages the dword of column
    // t % BN of the tile; it lands in LDS as [column] and every lane later picks its own.
    const uint32_t e_off = 4u * ((uint32_t)(min(strip0 + ((tid % C::BN) >> 4), L.nstrips - 1) * L.ngq * 16) + (tid & 15));
    // LDS byte addresses (the dynamic array is the kernel's only LDS object)
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)smem;
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
    auto advance = [&](GroupCursor& c) {
        const int sub = c.sub + 1;
        const bool wrap = sub == gq;
        c.sub = wrap ? 0 : sub;
        c.g += wrap ? 1 : 0;
    };

    // ---- one stage = NSIDE loads per wave: A_CHUNKS + B_CHUNKS 1 KB blocks and 256 B of exponents
    constexpr int NSIDE = C::A_CHUNKS + C::B_CHUNKS + 1;
    // t-th load of k-tile kt into LDS stage `stage`
    auto side_load = [&](int t, int kt, int stage, const GroupCursor& c) {
        const uint32_t st = (uint32_t)stage * C::STAGE;
        if (t < C::A_CHUNKS) lds_load16(a_base + kt * 128, a_off[t], st + a_dst + t * (kThreads / 64) * 1024);
        else if (t < C::A_CHUNKS + C::B_CHUNKS)
            lds_load16(b_base + (int64_t)kt * 1024, b_off[t - C::A_CHUNKS], st + b_dst + (t - C::A_CHUNKS) * (kThreads / 64) * 1024);
        else  // the dword holds 4 stored groups; the four 32-blocks of a k-tile always share one dword
            lds_load4(e_base + (group_of(c, kt, 0) >> 2) * 64, e_off, st + e_dst);
    };

    v4f acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    // ---- operand registers.  They are refilled in place: a weight fragment and its exponent dword
    // as soon as the last matrix instruction that reads them has been issued, the activation
    // fragment one row block ahead of its use.
    v8i bfr[WTN];
    uint32_t e_cur[WTN];
    // Activation fragments rotate through two registers sets: row block i multiplies one (fy for
    // even i, fz for odd i) while the next fragment arrives in the other.  In the exact mode the
    // multiplied set holds the lower exponent band and fx the upper one; the arriving fragment is
    // split in place, one dword per matrix instruction of the lower-band pass, into fx (whose old
    // content the upper-band pass has already consumed) and itself.
    v8i fx, fy, fz;
    GroupCursor cur_comp = {0, 0}, cur_load = {0, 0};
    // this lane's two 16-byte slots inside a 16-row sub-tile (rows of 128 B, chunks XOR-swizzled)
    const int a_rd0 = col * 128 + ((lb ^ (col & 7)) * 16), a_rd1 = col * 128 + ((lb ^ (col & 7) ^ 4) * 16);
    auto stage_a = [&](int stage) { return smem + stage * C::STAGE + (wm * WTM) * 2048; };
    auto stage_b = [&](int stage) { return smem + stage * C::STAGE + C::A_BYTES + (wn * WTN) * 1024 + lane * 16; };
    auto stage_e = [&](int stage) {
        return reinterpret_cast<const uint32_t*>(smem + stage * C::STAGE + C::A_BYTES + C::B_BYTES) + wn * WTN * 16 + col;
    };
    auto read_b = [&](int j, const uint8_t* sb, const uint32_t* se) {
        e_cur[j] = se[j * 16];  // raw dword: this lane's byte is shifted down at its first use
        const u32x4 b = *reinterpret_cast<const u32x4*>(sb + j * 1024);
        bfr[j] = (v8i){(int)b[0], (int)b[1], (int)b[2], (int)b[3], 0, 0, 0, 0};
    };
    auto read_a = [&](v8i& dst, const uint8_t* sub_tile) {
        const u32x4 p = *reinterpret_cast<const u32x4*>(sub_tile + a_rd0);
        const u32x4 q = *reinterpret_cast<const u32x4*>(sub_tile + a_rd1);
        dst = (v8i){(int)p[0], (int)p[1], (int)p[2], (int)p[3], (int)q[0], (int)q[1], (int)q[2], (int)q[3]};
    };
    auto split_in_place = [&](v8i& frag, int d) {  // dword d of frag -> upper band into fx, lower band stays
        uint32_t h, l;
        split_exponent_bands_dword((uint32_t)frag[d], h, l);
        fx[d] = (int)h;
        frag[d] = (int)l;
    };

    // ---- one k-step: the matrix instructions of k-tile kt on LDS stage `stage`.  In-order issue
    // means that whatever a wave puts between two matrix instructions runs in the shadow of the
    // matrix pipe, and whatever it puts after the last one waits for all of them; the scheduling
    // fences pin the order written here.  The step's barrier sits BEFORE its last row block: by then
    // every read of this stage has been issued (the last activation fragment is fetched one block
    // ahead), so behind the barrier the stage is free, and the next stage is complete.  The last
    // row block then carries, one per matrix instruction, the requests for k-tile kt + 3 into the
    // freed stage (LOAD) and the reads of the next step's first operands (NEXT): the matrix pipe
    // never waits for LDS at the top of a step.  WAIT is the number of this wave's loads that may
    // still be outstanding at the barrier (those of k-tile kt + 2).  The body has no branches.
    auto k_step = [&](int kt, int stage, auto load_tag, auto next_tag, auto wait_tag) {
        constexpr bool LOAD = decltype(load_tag)::value;
        constexpr bool NEXT = decltype(next_tag)::value;
        constexpr int WAIT = decltype(wait_tag)::value;
        const int stage_next = stage == C::NSTAGE - 1 ? 0 : stage + 1;
        const uint8_t* sa = stage_a(stage);
        const uint8_t* sa_next = stage_a(stage_next);
        const uint8_t* sb_next = stage_b(stage_next);
        const uint32_t* se_next = stage_e(stage_next);
        // this lane's exponent byte for each of its WTN columns: byte (stored group & 3) of the dword
        const int esh = 8 * (group_of(cur_comp, kt, lb) & 3);
        constexpr int PASSES = EXACT ? 2 : 1;
#pragma unroll
        for (int i = 0; i < WTM; ++i) {
            const bool last_block = i == WTM - 1;
            if (last_block && NEXT) {
                __builtin_amdgcn_sched_barrier(0);
                wait_loads_then_barrier<WAIT>();
                __builtin_amdgcn_sched_barrier(0);
            }
            v8i& cur = (i & 1) ? fz : fy;
            v8i& inc = (i & 1) ? fy : fz;
            const bool fetch = !last_block || NEXT;
            if (!last_block) read_a(inc, sa + (i + 1) * 2048);  // one block of matrix instructions ahead
            else if (NEXT) read_a(inc, sa_next);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
#pragma unroll
                for (int j = 0; j < WTN; ++j) {
                    const v8i& op = (EXACT && p == 0) ? fx : cur;
                    if (i == 0 && p == 0) e_cur[j] >>= esh;  // at its first use: the dword was the last thing read
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(op, bfr[j], acc[i][j], 0, 4, 0, 127, 0,
                                                                                  (int)e_cur[j]);
                    if (EXACT && p == 1 && fetch) {
#pragma unroll
                        for (int d = j * 8 / WTN; d < (j + 1) * 8 / WTN; ++d) split_in_place(inc, d);
                    }
                    if (last_block) {
                        const int t = p * WTN + j;  // position in the block's matrix-instruction stream
                        constexpr int PER = (NSIDE + WTN * PASSES - 1) / (WTN * PASSES);  // loads per slot
#pragma unroll
                        for (int q = 0; q < PER; ++q)
                            if (LOAD && t * PER + q < NSIDE) side_load(t * PER + q, kt + 3, stage, cur_load);
                        if (NEXT && p == PASSES - 1) read_b(j, sb_next, se_next);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        static_assert(WTM % 2 == 0 && 8 % WTN == 0, "fragment rotation and split slots assume these");
        advance(cur_comp);
        if (LOAD) advance(cur_load);
    };

    // ---- prologue: k-tiles 0, 1 and 2 into stages 0, 1 and 2; the first operands into registers
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
#pragma unroll
    for (int t = 0; t < NSIDE; ++t) side_load(t, 0, 0, cur_load);
    if (nkt > 1) {
        advance(cur_load);
#pragma unroll
        for (int t = 0; t < NSIDE; ++t) side_load(t, 1, 1, cur_load);
    }
    if (nkt > 2) {
        advance(cur_load);
#pragma unroll
        for (int t = 0; t < NSIDE; ++t) side_load(t, 2, 2, cur_load);
        advance(cur_load);  // now at k-tile 3
    }
    // k-tile 0 has landed, for every wave, once all but the later tiles' loads are done
    if (nkt > 2) wait_loads_then_barrier<2 * NSIDE>();
    else if (nkt > 1) wait_loads_then_barrier<NSIDE>();
    else wait_loads_then_barrier<0>();
    {
        const uint8_t* sb = stage_b(0);
        const uint32_t* se = stage_e(0);
        read_a(fy, stage_a(0));
#pragma unroll
        for (int j = 0; j < WTN; ++j) read_b(j, sb, se);
        if constexpr (EXACT) {
#pragma unroll
            for (int d = 0; d < 8; ++d) split_in_place(fy, d);
        }
    }

    // ---- main loop.  Step kt computes stage kt % 3; k-tiles kt + 1 and kt + 2 are in the other two
    // stages or on their way, k-tile kt + 3 is requested into stage kt % 3 behind the step's
    // barrier.  At that barrier each wave waits for all of its loads but the NSIDE of k-tile
    // kt + 2: then k-tile kt + 1 is complete once every wave is through, after two steps of slack
    // for the memory latency.  The last three steps request nothing and are peeled.
    using W1 = std::integral_constant<int, NSIDE>;
    using W0 = std::integral_constant<int, 0>;
    int stage = 0;
    auto next = [](int st) { return st == C::NSTAGE - 1 ? 0 : st + 1; };
    int kt = 0;
    for (; kt + 3 < nkt; ++kt) {
        k_step(kt, stage, yes{}, yes{}, W1{});
        stage = next(stage);
    }
    if (nkt > 2) {  // kt == nkt - 3: k-tile kt + 2 still outstanding
        k_step(kt, stage, no{}, yes{}, W1{});
        stage = next(stage);
        ++kt;
    }
    if (nkt > 1) {  // kt == nkt - 2
        k_step(kt, stage, no{}, yes{}, W0{});
        stage = next(stage);
        ++kt;
    }
    k_step(kt, stage, no{}, no{}, W0{});

    // ---- epilogue.  D[row][col] of a 16x16 tile sits in lane 16*(row/4)+col, register row%4:
    // good for the scale / LoRC arithmetic (one column per lane), bad for stores (64 B runs).
    // Each wave therefore passes its 16 x (16*WTN) slabs through a private LDS patch (row stride
    // 16*WTN + 4 floats: the four row groups of a store land on disjoint banks, rows stay 16 B
    // aligned) and writes them out as 16 B per lane, whole rows of the slab at a time.
    constexpr int SLAB_N = 16 * WTN, SLAB_LD = SLAB_N + 4;
    static_assert(C::THREADS / 64 * 16 * SLAB_LD * 4 <= C::NSTAGE * C::STAGE, "epilogue patch does not fit the stages");
    __syncthreads();  // every wave is done reading the stages
    float* patch = reinterpret_cast<float*>(smem) + wave * (16 * SLAB_LD);
    const float* colscale = reinterpret_cast<const float*>(blob + L.off_colscale);
    const int64_t n_wave = (strip0 + wn * WTN) * 16;
    float cn[WTN];
#pragma unroll
    for (int j = 0; j < WTN; ++j) cn[j] = colscale[min(n_wave + j * 16 + col, L.Np - 1)];
    constexpr int LPR = SLAB_N / 4;   // lanes per slab row when each lane carries 4 columns
    constexpr int RPI = 64 / LPR;     // slab rows per store instruction
    const int srow = lane / LPR, scol = (lane % LPR) * 4;
    const bool vec_ok = (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
#pragma unroll
    for (int i = 0; i < WTM; ++i) {
        const int64_t m_slab = m0 + (wm * WTM + i) * 16;
        float sxm[4];
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) sxm[rg] = sx[min(m_slab + 4 * lb + rg, M - 1)];
#pragma unroll
        for (int j = 0; j < WTN; ++j) {
            const int64_t n = min(n_wave + j * 16 + col, L.N - 1);
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float y = (sxm[rg] * cn[j]) * acc[i][j][rg];
                if (lorc.r > 0) {
                    const float* t = lorc.T + min(m_slab + 4 * lb + rg, M - 1) * lorc.r;
                    for (int q = 0; q < lorc.r; ++q) y = fmaf(t[q], half_bits_to_f32(lorc.V[(int64_t)q * L.N + n]), y);
                }
                patch[(4 * lb + rg) * SLAB_LD + j * 16 + col] = y;
            }
        }
#pragma unroll
        for (int t = 0; t < 16 / RPI; ++t) {
            const int r = t * RPI + srow;
            const v4f y = *reinterpret_cast<const v4f*>(patch + r * SLAB_LD + scol);
            const int64_t m = m_slab + r, n = n_wave + scol;
            if (m >= M || n >= L.N) continue;
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

template <int WTM, int WTN, int WAVES_M, int WAVES_N, bool EXACT>
hipError_t launch_cfg(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L, Lorc lorc,
                      void* Y, int64_t ldy, int out_dtype, hipStream_t s)
{
    using C = TileCfg<WTM, WTN, WAVES_M, WAVES_N>;
    const int tiles_m = (int)((M + C::BM - 1) / C::BM), tiles_n = (int)((L.Np + C::BN - 1) / C::BN);
    const int ntiles = tiles_m * tiles_n;
    const int per = (ntiles + 7) / 8;
    const size_t smem = C::NSTAGE * C::STAGE;
    auto kern = k_gemm_tile<WTM, WTN, WAVES_M, WAVES_N, EXACT>;
    static bool attr_done = false;  // raising the dynamic LDS limit is a per-function, per-process setting
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(C::THREADS), smem, s, Xq, sx, M, blob, L, lorc, Y, ldy,
                       out_dtype, tiles_m, tiles_n);
    return hipGetLastError();
}

template <bool EXACT>
hipError_t launch_pick(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L, Lorc lorc,
                       void* Y, int64_t ldy, int out_dtype, hipStream_t s)
{
    // 256 x 256 tiles once they fill the 256 compute units at least ~twice, else 128 x 128
    const int64_t big = ((M + 255) / 256) * ((L.Np + 255) / 256);
    if (big >= 384) return launch_cfg<4, 8, 4, 2, EXACT>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
    return launch_cfg<4, 4, 2, 2, EXACT>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
}

}  // namespace

bool gemm_tile_supported(int64_t M, const BlobLayout& L) { return M > 64 && L.N >= 64; }

hipError_t launch_gemm_tile(const uint8_t* Xq, const float* sx, int64_t M, const uint8_t* blob, const BlobLayout& L,
                            Lorc lorc, void* Y, int64_t ldy, int out_dtype, int accum, hipStream_t s)
{
    return accum == 0 ? launch_pick<true>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s)
                      : launch_pick<false>(Xq, sx, M, blob, L, lorc, Y, ldy, out_dtype, s);
}

}  // namespace zqfp
