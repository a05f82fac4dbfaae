// bf16 MFMA GEMM for gfx950:  C[M,N] (+)= A[M,K] * W[N,K]^T, f32 accumulate, with
//   - optional row gather on A and row grouping with per-group weights (top-2 MoE grouped GEMM),
//   - fused epilogues: f32 store, f32 residual accumulate, bf16 store, SwiGLU (two weight
//     matrices, silu(gate) * up, bf16 store).
//
// Design (64-wide wavefronts, CDNA4):
//   * workgroup = 4 wavefronts in a 2x2 grid; each wavefront owns a (16*MI) x (32*WN_T) block of
//     16x16 v_mfma_f32_16x16x32_bf16 tiles held in accumulator registers (measured on MI355X with
//     register-only operands: 2.41 PFLOP/s for this instruction, 2.04 for the 32x32x16 form).  The
//     weight fragment is the MFMA's A operand, so a lane ends up with four consecutive output
//     columns of one row and the epilogue stores 16 (f32) or 8 (bf16) bytes at a time;
//   * operands go global -> LDS with global_load_lds_dwordx4 (no VGPR staging), 64-wide K slabs, the
//     weights three slabs deep and the activations two (three where 160 KB allow).  A slab is two phases
//     (its two k-steps) with one barrier between them; the fragments of a k-step are read one phase
//     ahead; every LDS read and every direct-to-LDS load stands alone in front of one MFMA (a
//     compile-time list of micro-operations dealt over the MFMA slots), the loads issued from inline
//     assembly as scalar base + 32-bit lane offset and waited for with a counted vmcnt, the MFMAs issued
//     from assembly with their accumulators tied to registers (see the comments in gemm_tile for why
//     and what was measured);
//   * workgroups are persistent: one per compute unit, each walking its XCD's share of the tile list; the
//     last, partial round of tiles is cut into row halves when it would leave half the compute units idle;
//   * LDS rows are 128 B (64 bf16); the 16-byte chunk c of row r is stored at chunk position
//     c ^ ((r >> 1) & 7): the LDS serves a ds_read_b128 sixteen lanes (256 B, 64 banks) per cycle,
//     and 16 consecutive rows then cover all sixteen 16-byte bank groups (measured: the simpler
//     c ^ (r & 7) left every read 2-way conflicted).  Direct-to-LDS loads place lane i at
//     base + 16*i, so the swizzle is applied by choosing which global chunk a lane fetches;
//   * row tiles are balanced: r rows (of a group, or of the whole matrix) are cut into the fewest
//     tiles of at most `max_rows` rows, all of the same height (a multiple of 16), and the tile body
//     is instantiated for every accumulator height 32, 64, ... 256.  Equal tiles matter beyond the
//     saved padding: the row tiles of one (group, column tile) are dispatched back to back and run in
//     lockstep, so the weight slab one of them pulls from HBM is an L2 hit for the others (measured on
//     the MoE gate/up GEMM: with a full-tiles-plus-remainder split the short remainder tiles drift
//     ahead and the weights are fetched 2.7 times; with equal tiles 1.2 times);
//   * tile order: group (expert), then bands of four row tiles, then column tile, then row tile
//     within the band; the linear workgroup id is remapped so that each XCD (id % 8) walks one
//     contiguous range of that order: the ~32 workgroups an XCD runs at a time form a block of about
//     4 row tiles x 8 column tiles and share both operands in its L2 (measured on an 8192^3 product:
//     L2 hit rate 48 % -> 79 % against column-major tile order).
#include <algorithm>
#include <type_traits>
#include <utility>

#include "common.h"

// the direct-to-LDS loads below set M0 themselves and say so in their clobber list; clang notes that M0
// is a reserved register
#pragma clang diagnostic ignored "-Winline-asm"

namespace sv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

namespace {

template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>), ..., f(integral_constant<int, N-1>): a loop whose index is a compile-time constant
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

constexpr int BAND = 4;     // row tiles per band of the tile order

// r rows in the fewest tiles of at most max_rows rows (a multiple of 32, <= 256): nt tiles of rt
// rows each, rt a multiple of 16; the last tile takes what is left and may be shorter.
__host__ __device__ inline void split_rows(int r, int max_rows, int& nt, int& rt) {
    nt = (r + max_rows - 1) / max_rows;
    rt = nt > 0 ? (((r + nt - 1) / nt + 15) & ~15) : 0;
}

// One output tile with (32*MI) x (64*WN_T) accumulators: rows [row_begin, row_end) of the (gathered)
// A (row_end - row_begin <= 32*MI), output columns from n0 on, weights of `group`.
template <int MI, int WN_T, bool SWIGLU>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a, char* smem, int row_begin, int row_end, int n0,
                                          int group) {
    constexpr int BM = 32 * MI, BN = 64 * WN_T;
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;
    // LDS: activation stages, then three weight stages; the activations are three deep as well where
    // 160 KB allow it (tiles of up to 160 rows at 256 columns, every tile at 128 columns)
    constexpr int AST = 3 * (A_BYTES + B_BYTES) <= 160 * 1024 ? 3 : 2;
    constexpr int B_BASE = AST * A_BYTES;
    constexpr int A_INST = BM / 32, B_INST = BN / 32; // direct-to-LDS loads per wavefront per slab
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront id, kept in an SGPR
    const int wm = w >> 1, wn = w & 1;
    const char* Ab = (const char*)a.A;
    const char* Wb = (const char*)a.W + (int64_t)group * a.w_group_stride * 2;
    const char* W3b = SWIGLU ? (const char*)a.W3 + (int64_t)group * a.w_group_stride * 2 : nullptr;

    // ---- per-lane byte offsets of this lane's 16-byte chunks, relative to the (wave-uniform) operand
    // base: a load is "scalar base of the slab + this 32-bit offset", so advancing to the next slab costs
    // scalar adds only
    const int lrow = lane >> 3;                 // row inside an 8-row load group
    // swizzle key of tile row r is (r >> 1) & 7; load group q covers rows 8q..8q+7, so a lane's key
    // is (4q + lane/16) & 7 and it fetches global chunk (lane & 7) ^ key into slot lane & 7
    auto gchunk_of = [&](int q) { return (lane & 7) ^ ((4 * q + (lane >> 4)) & 7); };
    uint32_t a_o[A_INST], b_o[B_INST];
    // Source rows of this wavefront's activation loads.  With a row gather they come from memory: the loads
    // are issued here from assembly and waited for (by count) only behind the first weight loads of the
    // prologue, so that their latency runs beside that of the weights instead of in front of it (the
    // compiler would wait for them with a count that knows nothing of the assembly-issued loads).
    int srow[A_INST];
#pragma unroll
    for (int j = 0; j < A_INST; ++j) {
        int r = row_begin + (w * A_INST + j) * 8 + lrow;
        r = r < row_end ? r : row_end - 1;                       // clamp: masked at the store
        srow[j] = r;
        if (a.a_rows) {
            const int32_t* src = a.a_rows + r;
            asm volatile("global_load_dword %0, %1, off" : "=v"(srow[j]) : "v"(src) : "memory");
        }
    }
    const uint32_t w3_delta = SWIGLU ? (uint32_t)(W3b - Wb) : 0u;      // launcher: 0 < W3 - W < 2^31
#pragma unroll
    for (int j = 0; j < B_INST; ++j) {
        int tr = (w * B_INST + j) * 8 + lrow;                   // row of the B tile, 0..BN-1
        int n;
        uint32_t extra = 0;
        if (SWIGLU) {
            // a wavefront column block = [its gate features | the same up features]
            int wcol = tr / (BN / 2), within = tr % (BN / 2);
            bool up = within >= BN / 4;
            n = n0 + wcol * (BN / 4) + (up ? within - BN / 4 : within);
            extra = up ? w3_delta : 0u;
        } else {
            n = n0 + tr;
        }
        n = n < a.N ? n : a.N - 1;
        b_o[j] = (uint32_t)(((int64_t)n * a.K + gchunk_of(w * B_INST + j) * 8) * 2) + extra;
    }

    // Direct-to-LDS loads are issued from inline assembly (the compiler's wait-count pass would make every
    // fragment wait drain all LDS traffic behind a pending LDS-DMA load); their completion is waited for by
    // hand (vmcnt).  The LDS destination of lane i is M0 + 16 i.
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lds_ptr_t)smem);
    const uint32_t wu = (uint32_t)w;
    auto issue_a = [&](int q, int kt, int ast) {     // load q of activation slab kt into A stage ast
        const uint32_t dst = lds0 + ast * A_BYTES + (wu * A_INST + q) * 1024;
        const char* base = Ab + (int64_t)kt * 128;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(dst), "v"(a_o[q]), "s"(base) : "memory", "m0");
    };
    auto issue_b = [&](int q, int kt, int bst) {     // load q of weight slab kt into B stage bst
        const uint32_t dst = lds0 + B_BASE + bst * B_BYTES + (wu * B_INST + q) * 1024;
        const char* base = Wb + (int64_t)kt * 128;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(dst), "v"(b_o[q]), "s"(base) : "memory", "m0");
    };

    constexpr int NI = 2 * WN_T;              // 16x16 tiles per wavefront: MI rows x NI columns
    f32x4_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    // fragment read offsets: row (lane & 15) of each 16-row tile, chunk (4*kk + lane/16) ^ key(row)
    const int frag_row = lane & 15, kquart = lane >> 4, sw = (frag_row >> 1) & 7;
    const int a_off = (wm * 16 * MI + frag_row) * 128;
    const int b_off = (wn * 32 * WN_T + frag_row) * 128;

    constexpr int NL = A_INST + B_INST;      // slab loads per wavefront
    constexpr int NM = MI * NI;              // MFMAs of one k-step
    constexpr int NR = MI + NI;              // fragment reads of one k-step

    // Pipeline.  A slab (64 of K) is two phases, k-step 0 and k-step 1, of NM MFMAs each, with ONE
    // barrier per slab between them.  The MFMA pipe takes a new instruction every 16 cycles and the
    // wavefront issues in order, so whatever sits between two MFMAs must issue within the ~12 cycles the
    // pipe is still busy or it opens a bubble (measured: the 16 fragment reads or the 8 loads of a
    // k-step issued as a group cost ~110 cycles of MFMA time each, 10 % per group).  Every phase therefore
    // issues its memory instructions ONE per MFMA slot, alternating fragment reads and loads:
    //   phase 0 of slab kt multiplies k-step 0 (fragments read during phase 1 of slab kt-1), reads the
    //     k-step-1 fragments of slab kt and issues the weight loads of slab kt+2;
    //   then the wavefront waits for its own loads of slab kt+1 (vmcnt) and for its fragment reads, and
    //     all wavefronts meet: slab kt has been read by everyone, slab kt+1 has landed;
    //   phase 1 multiplies k-step 1, reads the k-step-0 fragments of slab kt+1 and issues the activation
    //     loads of slab kt+AST into the stage slab kt just left.
    // No MFMA waits for a read issued right in front of it, and the barrier comes when a wavefront's
    // reads are long complete.
    const int KT = a.K / 64;
    bf16x8_t af[2][MI], bfr[2][NI];
    auto stage_a = [&](int kt) { return smem + (AST == 3 ? kt % 3 : kt & 1) * A_BYTES; };
    auto stage_b = [&](int kt) { return smem + B_BASE + (kt % 3) * B_BYTES; };
    // fragment read r of k-step kk of a slab: the weight fragments first (the first row of MFMAs needs all
    // of them), then the activation fragments in row order
    auto read_frag = [&](const char* As, const char* Bs, int kk, int r) {
        const int coff = ((4 * kk + kquart) ^ sw) << 4;
        if (r < NI) bfr[kk][r] = *(const bf16x8_t*)(Bs + b_off + r * 16 * 128 + coff);
        else af[kk][r - NI] = *(const bf16x8_t*)(As + a_off + (r - NI) * 16 * 128 + coff);
    };
    auto wait_vm = [&](auto n_c) {          // vmcnt(n) and lgkmcnt(0)
        constexpr int N = decltype(n_c)::value;
        __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
    };
    using I0 = std::integral_constant<int, 0>;
    // loads that may stay pending at the barrier of slab kt: those issued for slab kt+2
    using IB = std::integral_constant<int, AST == 3 ? NL : B_INST>;
    using IPRO = std::integral_constant<int, (AST - 1) * A_INST>;

    // prologue: weights of slabs 0 and 1, then (their source rows have arrived) activations of slabs
    // 0..AST-1.  Loads land in issue order: at the first barrier only activations of later slabs may be
    // pending.
#pragma unroll
    for (int q = 0; q < B_INST; ++q) issue_b(q, 0, 0);
    if (KT > 1) {
#pragma unroll
        for (int q = 0; q < B_INST; ++q) issue_b(q, 1, 1);
    }
    if (a.a_rows) {
        if (KT > 1) asm volatile("s_waitcnt %0" :: "n"(0x0070 | ((2 * B_INST) & 15) | (((2 * B_INST) >> 4) << 14)) : "memory");
        else asm volatile("s_waitcnt %0" :: "n"(0x0070 | (B_INST & 15) | ((B_INST >> 4) << 14)) : "memory");
    }
#pragma unroll
    for (int j = 0; j < A_INST; ++j) {
        asm volatile("" : "+v"(srow[j]));         // (used only behind the wait above)
        a_o[j] = (uint32_t)(((int64_t)srow[j] * a.lda + gchunk_of(w * A_INST + j) * 8) * 2);
    }
#pragma unroll
    for (int q = 0; q < A_INST; ++q) issue_a(q, 0, 0);
    if (KT > 1) {
#pragma unroll
        for (int q = 0; q < A_INST; ++q) issue_a(q, 1, 1);
        if (AST == 3 && KT > 2) {
#pragma unroll
            for (int q = 0; q < A_INST; ++q) issue_a(q, 2, 2);
        }
    }
    if (KT > 1 && (KT > 2 || AST == 2)) wait_vm(IPRO{}); else wait_vm(I0{});
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < NR; ++r) read_frag(stage_a(0), stage_b(0), 0, r);

    // One phase: NM MFMAs of k-step KK with n_rd fragment reads (k-step RK of the slab at As/Bs) and n_ld
    // loads spread over the MFMA slots.  Micro-op k of the merged list (read, load, read, load, ... then
    // what is left of the longer list) goes in front of MFMA floor(k * NM / n_ops).
    auto phase = [&](auto kk_c, auto n_rd_c, auto n_ld_c, auto&& read_op, auto&& load_op, auto&& m0_op) {
        constexpr int KK = decltype(kk_c)::value;
        constexpr int N_RD = decltype(n_rd_c)::value, N_LD = decltype(n_ld_c)::value;
        constexpr int N_OPS = N_RD + N_LD;
        constexpr int N_PAIR = N_RD < N_LD ? N_RD : N_LD;
        // position of load j in the merged list, and the MFMA slot of list position k
        auto k_of_load = [](int j) constexpr { return j < N_PAIR ? 2 * j + 1 : j + N_PAIR; };
        auto slot_of = [](int k) constexpr { return k * NM / (N_OPS > 0 ? N_OPS : 1); };
        // M0 of the phase's first load: an MFMA separates it from the load unless the load sits in slot 0
        if constexpr (N_LD > 0) m0_op(std::integral_constant<int, 0>{}, std::integral_constant<bool, slot_of(k_of_load(0)) == 0>{});
        static_for<NM>([&](auto m_c) {
            constexpr int m = decltype(m_c)::value;
            // micro-ops k with floor(k * NM / N_OPS) == m
            constexpr int k0 = (m * N_OPS + NM - 1) / NM, k1 = ((m + 1) * N_OPS + NM - 1) / NM;
            static_for<k1 - k0>([&](auto d_c) {
                constexpr int k = k0 + decltype(d_c)::value;
                constexpr bool is_rd = k < 2 * N_PAIR ? (k & 1) == 0 : (N_RD > N_LD);
                constexpr int idx = k < 2 * N_PAIR ? (k >> 1) : k - N_PAIR;
                if constexpr (is_rd) read_op(std::integral_constant<int, idx>{});
                else {
                    load_op(std::integral_constant<int, idx>{});
                    // M0 of the next load goes out right behind this one: the MFMAs up to that load's slot
                    // are the wait state the hardware wants between an M0 write and its use
                    if constexpr (idx + 1 < N_LD)
                        m0_op(std::integral_constant<int, idx + 1>{},
                              std::integral_constant<bool, slot_of(k_of_load(idx + 1)) == slot_of(k)>{});
                }
            });
            __builtin_amdgcn_sched_barrier(0);
            // (assembly with the accumulator tied to its register tuple: with one scheduling region per MFMA
            // the register allocator otherwise splits the accumulators between the two register files and
            // copies them back and forth every slab.)  The first 48 accumulator tiles live in AGPRs (192 of
            // the 256), any further ones (a 256-row tile has 64) in VGPRs.
            constexpr int i = m / NI, j = m % NI;
            if constexpr (m < 48)
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(bfr[KK][j]), "v"(af[KK][i]));
            else
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i][j]) : "v"(bfr[KK][j]), "v"(af[KK][i]));
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using CNR = std::integral_constant<int, NR>;
    using CA = std::integral_constant<int, A_INST>;
    using CB = std::integral_constant<int, B_INST>;

    // one slab; MORE2: slab kt+2 exists (its weights are issued in phase 0), MOREA: slab kt+AST exists (its
    // activations are issued in phase 1), NEXT: slab kt+1 exists
    auto body = [&](int kt, auto more2_c, auto morea_c, auto next_c) {
        constexpr bool MORE2 = decltype(more2_c)::value, MOREA = decltype(morea_c)::value, NEXT = decltype(next_c)::value;
        const int bst2 = (kt + 2) % 3;
        const char* As0 = stage_a(kt); const char* Bs0 = stage_b(kt);
        auto no_m0 = [](auto, auto) {};
        phase(C0{}, CNR{}, std::integral_constant<int, MORE2 ? B_INST : 0>{},
              [&](auto r_c) { read_frag(As0, Bs0, 1, decltype(r_c)::value); },
              [&](auto q_c) { issue_b(decltype(q_c)::value, kt + 2, bst2); }, no_m0);
        if (MORE2) wait_vm(IB{}); else wait_vm(I0{});
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const int ast2 = AST == 3 ? (kt + AST) % 3 : (kt + AST) & 1;
        const char* As1 = stage_a(kt + 1); const char* Bs1 = stage_b(kt + 1);
        phase(C1{}, std::integral_constant<int, NEXT ? NR : 0>{}, std::integral_constant<int, MOREA ? A_INST : 0>{},
              [&](auto r_c) { read_frag(As1, Bs1, 0, decltype(r_c)::value); },
              [&](auto q_c) { issue_a(decltype(q_c)::value, kt + AST, ast2); }, no_m0);
    };

    // The steady state with every stage index a compile-time constant (slab s of a period of PER slabs):
    // a fragment read is one ds_read_b128 from a per-lane base register (one per stage and k-step, kept
    // for the whole loop) plus an immediate, a load is "M0 = scalar base + immediate" and the load itself,
    // and nothing is left of the stage arithmetic.  With one wavefront per SIMD every instruction the
    // wavefront issues between two MFMAs takes issue time from them (about 4 cycles each, measured: a slab
    // of 96 MFMAs with 132 other instructions took 1536 + 4 x 132 cycles), so the instruction count of the
    // loop is what separates it from the MFMA rate.
    constexpr int PER = AST == 3 ? 3 : 6;
    typedef const __attribute__((address_space(3))) char* lds_cptr;
    lds_cptr a_rd[AST][2], b_rd[3][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int coff = ((4 * kk + kquart) ^ sw) << 4;
#pragma unroll
        for (int st = 0; st < AST; ++st) a_rd[st][kk] = (lds_cptr)smem + st * A_BYTES + a_off + coff;
#pragma unroll
        for (int st = 0; st < 3; ++st) b_rd[st][kk] = (lds_cptr)smem + B_BASE + st * B_BYTES + b_off + coff;
    }
    const uint32_t a_ld0 = lds0 + wu * A_INST * 1024, b_ld0 = lds0 + B_BASE + wu * B_INST * 1024;
    auto body_s = [&](auto s_c, int kt) {
        constexpr int S = decltype(s_c)::value;
        constexpr int SA0 = AST == 3 ? S % 3 : S & 1, SB0 = S % 3;                       // stages of slab kt
        constexpr int SA1 = AST == 3 ? (S + 1) % 3 : (S + 1) & 1, SB1 = (S + 1) % 3;       // of slab kt+1
        constexpr int SB2 = (S + 2) % 3, SA2 = AST == 3 ? (S + AST) % 3 : (S + AST) & 1;   // where the loads go
        typedef const __attribute__((address_space(3))) bf16x8_t* lds_frag;
        const char* wbase = Wb + (int64_t)(kt + 2) * 128;
        const char* abase = Ab + (int64_t)(kt + AST) * 128;
        phase(C0{}, CNR{}, CB{},
              [&](auto r_c) {
                  constexpr int r = decltype(r_c)::value;
                  if constexpr (r < NI) bfr[1][r] = *(lds_frag)(b_rd[SB0][1] + r * 2048);
                  else af[1][r - NI] = *(lds_frag)(a_rd[SA0][1] + (r - NI) * 2048);
              },
              [&](auto q_c) {
                  // (locals: operands of an assembly statement do not make a generic lambda capture a variable)
                  const uint32_t off = b_o[decltype(q_c)::value];
                  const char* base = wbase;
                  asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(off), "s"(base) : "memory");
              },
              [&](auto q_c, auto nop_c) {
                  constexpr int off = SB2 * B_BYTES + decltype(q_c)::value * 1024;
                  const uint32_t base = b_ld0;
                  if constexpr (decltype(nop_c)::value) asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0" :: "s"(base), "n"(off) : "m0", "scc");
                  else asm volatile("s_add_u32 m0, %0, %1" :: "s"(base), "n"(off) : "m0", "scc");
              });
        wait_vm(IB{});
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        phase(C1{}, CNR{}, CA{},
              [&](auto r_c) {
                  constexpr int r = decltype(r_c)::value;
                  if constexpr (r < NI) bfr[0][r] = *(lds_frag)(b_rd[SB1][0] + r * 2048);
                  else af[0][r - NI] = *(lds_frag)(a_rd[SA1][0] + (r - NI) * 2048);
              },
              [&](auto q_c) {
                  const uint32_t off = a_o[decltype(q_c)::value];
                  const char* base = abase;
                  asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(off), "s"(base) : "memory");
              },
              [&](auto q_c, auto nop_c) {
                  constexpr int off = SA2 * A_BYTES + decltype(q_c)::value * 1024;
                  const uint32_t base = a_ld0;
                  if constexpr (decltype(nop_c)::value) asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0" :: "s"(base), "n"(off) : "m0", "scc");
                  else asm volatile("s_add_u32 m0, %0, %1" :: "s"(base), "n"(off) : "m0", "scc");
              });
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    int kt = 0;
    // whole periods while the three slabs behind them still load everything (kt stays a multiple of PER)
    for (; kt + PER + 2 < KT; kt += PER) static_for<PER>([&](auto s_c) { body_s(s_c, kt + decltype(s_c)::value); });
    for (; kt + 3 < KT; ++kt) body(kt, T_{}, T_{}, T_{});
    // the last three slabs (fewer if the product is that short)
    if (kt + 2 < KT) {                       // slab KT-3: weights of the last slab; its activations only if two stages
        if (AST == 2) body(kt, T_{}, T_{}, T_{}); else body(kt, T_{}, F_{}, T_{});
        ++kt;
    }
    if (kt + 1 < KT) { body(kt, F_{}, F_{}, T_{}); ++kt; }
    if (kt < KT) body(kt, F_{}, F_{}, F_{});
    // the last MFMAs must have left the pipe before the accumulators are read (the compiler cannot see the
    // producers inside the assembly statements)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

    // ---- epilogue: tile (i, j) of a lane: output row i*16 + (lane & 15), columns j*16 + 4*(lane/16)
    // + 0..3 (the weight fragment was the A operand), stored as one 16- or 8-byte vector; the launcher
    // guarantees N and the row pitch are multiples of 4.
    int row_in = lane & 15, cq = (lane >> 4) * 4;
    // (passed through an empty assembly statement behind the main loop: the compiler otherwise computes the
    // epilogue's per-row addresses ahead of the loop and spills them to carry them across it)
    asm volatile("" : "+v"(row_in), "+v"(cq));
    if constexpr (SWIGLU) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int row = row_begin + wm * 16 * MI + i * 16 + row_in;
#pragma unroll
            for (int j = 0; j < NI / 2; ++j) {
                const int col = n0 + wn * (BN / 4) + j * 16 + cq;
                f32x4_t g = acc[i][j], u = acc[i][j + NI / 2], p;
#pragma unroll
                for (int r = 0; r < 4; ++r) p[r] = g[r] * __builtin_amdgcn_rcpf(1.0f + __expf(-g[r])) * u[r];   // (1 ulp reciprocal)
                if (row < row_end && col < a.N)
                    *(bf16x4_t*)((bf16*)a.C + (int64_t)row * a.ldc + col) = __builtin_convertvector(p, bf16x4_t);
            }
        }
    } else {
        auto store_all = [&](auto kind) {
            constexpr int KIND = decltype(kind)::value;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int row = row_begin + wm * 16 * MI + i * 16 + row_in;
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int col = n0 + wn * 32 * WN_T + j * 16 + cq;
                    if (row >= row_end || col >= a.N) continue;
                    const int64_t o = (int64_t)row * a.ldc + col;
                    if constexpr (KIND == EPI_STORE_F32) *(f32x4_t*)((float*)a.C + o) = acc[i][j];
                    else if constexpr (KIND == EPI_ADD_F32) {
                        f32x4_t* d = (f32x4_t*)((float*)a.C + o);
                        *d = *d + acc[i][j];
                    } else *(bf16x4_t*)((bf16*)a.C + o) = __builtin_convertvector(acc[i][j], bf16x4_t);
                }
            }
        };
        if (a.epilogue == EPI_ROPE_KV) {
            // QKV projection: this wavefront's 128 columns are one head (BN = 256, head_dim 128); the
            // rotation partner of dim j*16 + c is dim (j + 4)*16 + c, i.e. tile j + 4 of the same lane
            if constexpr (WN_T == 4) {
                const RopeKvArgs& rp = a.rope;
                const int head = (n0 + wn * 128) >> 7;                 // wave-uniform
                const int Hq = rp.n_q_heads, Hkv = rp.geom.n_kv_heads;
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int row = row_begin + wm * 16 * MI + i * 16 + row_in;
                    if (row >= row_end || head >= Hq + 2 * Hkv) continue;
                    // where this row's 128 values of the head go: the q buffer, or the row's slot of a KV page
                    // (one pair of 16-column tiles at a time, so that few values are live at once)
                    const bool is_q = head < Hq, is_k = !is_q && head < Hq + Hkv;
                    bf16* dst = nullptr;
                    bf16* kvp = (bf16*)rp.kv_layer;
                    int64_t page = 0;
                    int slot = 0, kvh = 0;
                    if (is_q) {
                        dst = (bf16*)rp.q_out + ((int64_t)row * Hq + head) * 128;
                    } else {
                        const int pos = rp.row_pos[row];
                        if (pos < 0) continue;
                        const int lp = pos / rp.geom.page_tokens;
                        if (lp >= rp.geom.pages_per_seq) continue;
                        page = rp.page_table[(row / rp.n_new) * rp.geom.pages_per_seq + lp];
                        slot = pos % rp.geom.page_tokens;
                        if (is_k) dst = kvp + rp.geom.k_off(page, head - Hq, slot);
                        else kvh = head - Hq - Hkv;
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        f32x4_t lo = acc[i][j], hi = acc[i][j + 4];
                        if (is_q || is_k) {
                            const float2* cp = rp.cs + (int64_t)row * 64 + j * 16 + cq;
                            const f32x4_t c01 = *(const f32x4_t*)cp, c23 = *(const f32x4_t*)(cp + 2);
                            const float cs_c[4] = {c01[0], c01[2], c23[0], c23[2]};
                            const float cs_s[4] = {c01[1], c01[3], c23[1], c23[3]};
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float x0 = lo[r], x1 = hi[r];
                                lo[r] = x0 * cs_c[r] - x1 * cs_s[r];
                                hi[r] = x1 * cs_c[r] + x0 * cs_s[r];
                            }
                            *(bf16x4_t*)(dst + j * 16 + cq) = __builtin_convertvector(lo, bf16x4_t);
                            *(bf16x4_t*)(dst + 64 + j * 16 + cq) = __builtin_convertvector(hi, bf16x4_t);
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                kvp[rp.geom.v_off(page, kvh, slot, j * 16 + cq + r)] = f32_to_bf16(lo[r]);
                                kvp[rp.geom.v_off(page, kvh, slot, 64 + j * 16 + cq + r)] = f32_to_bf16(hi[r]);
                            }
                        }
                    }
                }
            }
        } else if (a.epilogue == EPI_STORE_F32) store_all(std::integral_constant<int, EPI_STORE_F32>{});
        else if (a.epilogue == EPI_ADD_F32) store_all(std::integral_constant<int, EPI_ADD_F32>{});
        else store_all(std::integral_constant<int, EPI_STORE_T>{});
    }
}

// position `local` of a group's nt x tiles_n tiles, ordered band of BAND row tiles, then column tile,
// then row tile within the band
__device__ inline void band_order(int local, int nt, int tiles_n, int& tile_m, int& tile_n) {
    const int per_band = BAND * tiles_n;
    const int band = local / per_band, in_band = local % per_band;
    const int first = band * BAND;
    const int bm = nt - first < BAND ? nt - first : BAND;
    tile_n = in_band / bm;
    tile_m = first + in_band % bm;
}

// dynamic LDS a launch needs: the largest of activation stages + three weight stages over the tile heights
// (the same stage rule as in gemm_tile)
template <int BN>
constexpr int gemm_lds_bytes() {
    int need = 0;
    for (int mi = 1; mi <= 8; ++mi) {
        const int a_bytes = 32 * mi * 128, b_bytes = BN * 128;
        const int ast = 3 * (a_bytes + b_bytes) <= 160 * 1024 ? 3 : 2;
        const int n = ast * a_bytes + 3 * b_bytes;
        need = n > need ? n : need;
    }
    return need;
}

constexpr int MAX_GROUPS_FAST = 63;   // group offsets are fetched by one load (lane g holds offset g)
constexpr int CUS_PER_XCD = 32;

template <int WN_T, bool SWIGLU>
__global__ void __launch_bounds__(256, 1)
gemm_bf16_mfma_kernel(GemmArgs a, int max_rows, int tiles_n) {
    constexpr int BN = 64 * WN_T;
    constexpr int N_OUT = SWIGLU ? BN / 2 : BN;       // output columns per workgroup
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // ---- which tile.  Workgroup id x runs on XCD x % 8, and each XCD takes one contiguous range of the
    // logical tile order (see the head of this file).  The group offsets come from ONE load (lane g
    // fetches offset g; read back lane by lane): walking them one dependent load after the other cost
    // 3.6 us per workgroup, 4 % of a MoE tile.
    const int lane = threadIdx.x & 63;
    const int ng = a.group_offsets ? a.n_groups : 0;
    // Lane g of every wavefront keeps group g's row range, its split into row tiles and the position of
    // its first tile in the logical order; a tile finds its group with one ballot and reads the lane.
    // (Walking the groups with two integer divisions each cost about 4 us per tile, 5 % of a MoE tile.)
    int g_b0 = 0, g_b1 = 0, g_nt = 0, g_rt = 0, g_base = 0;
    int g_cnt = 0, g_cost = 0, g_work = 0;     // tiles of the group, cost of one column of its row tiles, work before it
    int total = 0, total_work = 0;
    if (ng > 0) {
        g_b0 = a.group_offsets[lane < ng ? lane : ng];
        g_b1 = a.group_offsets[lane + 1 < ng ? lane + 1 : ng];
        split_rows(lane < ng ? g_b1 - g_b0 : 0, max_rows, g_nt, g_rt);
        g_cnt = g_nt * tiles_n;
        // a tile of accumulator height MI (32-row units) costs about 4 MI + 5 (measured on the MoE gate/up
        // product: tiles of 7 units take 1.134 times as long as tiles of 6; the constant is the part of a
        // slab that does not grow with the height); the last row tile of a group may be lower than the rest
        if (g_nt > 0) {
            const int last_rows = (g_b1 - g_b0) - (g_nt - 1) * g_rt;
            g_cost = (g_nt - 1) * (4 * ((g_rt + 31) >> 5) + 5) + 4 * ((last_rows + 31) >> 5) + 5;
        }
        const int mine_w = tiles_n * g_cost;
        for (int g = 0; g < ng; ++g) {
            if (lane == g) { g_base = total; g_work = total_work; }
            total += __builtin_amdgcn_readlane(g_cnt, g);
            total_work += __builtin_amdgcn_readlane(mine_w, g);
        }
        if (lane >= ng) { g_base = 0x7fffffff; g_work = 0x7fffffff; }
    } else {
        int nt, rt;
        split_rows(a.M, max_rows, nt, rt);
        total = nt * tiles_n;
    }
    // An XCD's range is dealt to its 32 compute units one tile at a time (workgroups start in id order as
    // units fall free).  When the last round would occupy at most half the units, each of its tiles is
    // cut into two row halves that run as two workgroups: every unit then gets the same amount of work
    // (the MoE gate/up product is 10.5 rounds of tiles: without the cut half the units idle through the
    // eleventh, 9 % of the kernel).
    //
    // The workgroups are persistent: the grid is one workgroup per compute unit (fewer for small products),
    // and workgroup s of an XCD runs slots s, s + W, s + 2W, ... of the XCD's list (W workgroups per XCD), the
    // order in which the hardware would have started one workgroup per tile.  Looking up the group offsets,
    // starting and retiring a workgroup cost 3.6 us per tile (4 % of a MoE tile) when every tile was a
    // workgroup of its own.
    //
    // Which tiles an XCD takes.  A single matrix: equal shares of the tile list.  A grouped product: the
    // groups have different row counts, hence tiles of different heights, and an XCD's share is a
    // contiguous range of equal WORK (estimated from the tiles' accumulator heights): with equal tile counts each
    // XCD had exactly one expert of the MoE products and the kernel took as long as the largest expert
    // (workgroup lifetimes 881-1039 us, mean 942, on the gate/up product).  Tile t belongs to the XCD in
    // whose eighth of the total work its midpoint falls.
    const int xcd = (int)(blockIdx.x & 7);
    int per_xcd = (total + 7) >> 3, my_start = xcd * per_xcd;
    if (ng > 0) {
        auto start_of = [&](int x) -> int {              // first tile of XCD x's range
            if (x >= 8) return total;
            const long long t8 = (long long)x * total_work;                  // 8 x the work in front of the range
            const int grp = __builtin_popcountll(__ballot(8ll * g_work <= t8)) - 1;
            const int wb = __builtin_amdgcn_readlane(g_work, grp), c = __builtin_amdgcn_readlane(g_cost, grp);
            const int n = __builtin_amdgcn_readlane(g_cnt, grp), b = __builtin_amdgcn_readlane(g_base, grp);
            const int nt = __builtin_amdgcn_readlane(g_nt, grp);
            if (n == 0 || c == 0) return b;
            // a tile of the group costs c / nt on average (the order alternates its row tiles): tile j has its
            // midpoint at wb + (j + 1/2) c / nt; the first j with 8 x that >= t8
            const long long num = 2 * (t8 - 8ll * wb) * nt - 8ll * c, den = 16ll * c;
            const long long j0 = num <= 0 ? 0 : (num + den - 1) / den;
            return b + (int)(j0 < n ? j0 : n);
        };
        my_start = start_of(xcd);
        per_xcd = start_of(xcd + 1) - my_start;
    }
    const int rem = per_xcd % CUS_PER_XCD;
    const int n_split = (per_xcd > CUS_PER_XCD && rem > 0 && rem <= CUS_PER_XCD / 2) ? rem : 0;
    const int wg_per_xcd = (int)(gridDim.x >> 3);
    for (int slot = (int)(blockIdx.x >> 3); slot < per_xcd + n_split; slot += wg_per_xcd) {
    int t = slot, half = -1;
    if (slot >= per_xcd - n_split) {
        const int s2 = slot - (per_xcd - n_split);
        t = per_xcd - n_split + (s2 >> 1);
        half = s2 & 1;
    }
    const int logical = my_start + t;
    if (logical >= total) break;            // (slots grow with the loop: every later one is past the end too)
    int tile_m = 0, tile_n = 0, row_begin = 0, row_end = 0, group = 0;
    if (ng > 0) {
        // the last group whose first tile is not behind this one (groups without rows share their
        // successor's position and are passed over)
        group = __builtin_popcountll(__ballot(g_base <= logical)) - 1;
        const int b0 = __builtin_amdgcn_readlane(g_b0, group), b1 = __builtin_amdgcn_readlane(g_b1, group);
        const int nt = __builtin_amdgcn_readlane(g_nt, group), rt = __builtin_amdgcn_readlane(g_rt, group);
        band_order(logical - __builtin_amdgcn_readlane(g_base, group), nt, tiles_n, tile_m, tile_n);
        row_begin = b0 + tile_m * rt;
        row_end = row_begin + rt < b1 ? row_begin + rt : b1;
    } else {
        int nt, rt;
        split_rows(a.M, max_rows, nt, rt);
        band_order(logical, nt, tiles_n, tile_m, tile_n);
        row_begin = tile_m * rt;
        row_end = row_begin + rt < a.M ? row_begin + rt : a.M;
    }
    if (half >= 0) {                // a row half of a tile of the last round (halves of a multiple of 16 rows)
        const int mid = row_begin + ((((row_end - row_begin + 1) >> 1) + 15) & ~15);
        if (half == 0) row_end = mid < row_end ? mid : row_end;
        else row_begin = mid;
    }
    const int rows = row_end - row_begin;
    if (rows <= 0) continue;        // rounding the tile height up to 16 can leave a last tile (or half) empty
    const int n0 = tile_n * N_OUT;
    switch ((rows + 31) >> 5) {
        case 1: gemm_tile<1, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        case 2: gemm_tile<2, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        case 3: gemm_tile<3, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        case 4: gemm_tile<4, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        case 5: gemm_tile<5, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        case 6: gemm_tile<6, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        case 7: gemm_tile<7, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
        default: gemm_tile<8, WN_T, SWIGLU>(a, smem, row_begin, row_end, n0, group); break;
    }
    // (no barrier between tiles: behind the last barrier of a tile no wavefront reads LDS any more, so the
    // next tile's first loads may overwrite the stages at once)
    }
}

template <int WN_T, bool SWIGLU>
hipError_t launch_cfg(const GemmArgs& a, int max_rows, hipStream_t st) {
    constexpr int BN = 64 * WN_T;
    constexpr int N_OUT = SWIGLU ? BN / 2 : BN;
    // what the tallest need of any tile height is: gemm_tile keeps three activation stages where three of
    // each operand fit into 160 KB and two otherwise (with 128-column tiles every height has three: 144 KB
    // at 256 rows, which a size computed for two stages does not cover)
    constexpr int SMEM = gemm_lds_bytes<BN>();
    static_assert(SMEM <= 160 * 1024, "LDS of a compute unit");
    static bool attr_set = false;
    auto kern = gemm_bf16_mfma_kernel<WN_T, SWIGLU>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_n = (a.N + N_OUT - 1) / N_OUT;
    int tiles_m;
    if (a.group_offsets) {
        // every group rounds its tile count up, so at most n_groups more row tiles than rows / max_rows
        tiles_m = (a.m_upper + max_rows - 1) / max_rows + a.n_groups;
    } else {
        int rt;
        split_rows(a.M, max_rows, tiles_m, rt);
    }
    // one workgroup per compute unit (the LDS of a unit holds one), fewer if there are fewer tiles
    const int per_xcd = std::min((tiles_m * tiles_n + 7) / 8, CUS_PER_XCD);
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(256), SMEM, st, a, max_rows, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_mfma_bf16(const GemmArgs& a, hipStream_t st) {
    const int rows = a.group_offsets ? a.m_upper : a.M;
    if (rows <= 0 || a.N <= 0) return hipSuccess;
    // the MFMA path needs whole 64-wide K slabs, 16-byte aligned operand rows and output rows that
    // take 4-element vector stores; anything else (never the case for the supported model shapes)
    // takes the plain kernel
    if (a.K % 64 != 0 || a.lda % 8 != 0 || ((uintptr_t)a.A & 15) || ((uintptr_t)a.W & 15) || a.N % 4 != 0 ||
        a.ldc % 4 != 0 || ((uintptr_t)a.C & 15) || (a.epilogue == EPI_SWIGLU_T && ((uintptr_t)a.W3 & 15)))
        return a.epilogue == EPI_ROPE_KV ? hipErrorInvalidValue : launch_gemm_simple(a, SPEC_BF16, st);
    const bool sw = a.epilogue == EPI_SWIGLU_T;
    // operand rows are addressed as a 64-bit base per slab plus a 32-bit byte offset per lane: the rows a
    // launch can touch must lie within 4 GB of the operand's base (the up matrix of a SwiGLU product within
    // 2 GB above its gate matrix), and the fast group-offset fetch holds at most 63 groups
    {
        const int64_t a_rows_max = a.a_rows ? std::max<int64_t>(a.m_upper, a.M) : a.M;   // gathered rows are < m_upper
        const int64_t w3d = sw ? ((const char*)a.W3 - (const char*)a.W) : 0;
        if (a_rows_max * a.lda * 2 >= (int64_t)1 << 32 || (int64_t)a.N * a.K * 2 + w3d >= (int64_t)1 << 32 || w3d < 0 ||
            w3d >= (int64_t)1 << 31 || (a.group_offsets && a.n_groups > MAX_GROUPS_FAST))
            return a.epilogue == EPI_ROPE_KV ? hipErrorInvalidValue : launch_gemm_simple(a, SPEC_BF16, st);
    }
    if (a.epilogue == EPI_ROPE_KV && (a.group_offsets || a.rope.geom.head_dim != 128 || a.N % 128 != 0))
        return hipErrorInvalidValue;
    // Tile height: the one whose tile count fills the 256 compute units best.  The cost of a tile is
    // its accumulator height in 32-row units plus about three units for the column operand and the
    // per-slab overheads (fitted to measurements of the projection shapes).  Grouped problems are
    // judged by their average group (the group sizes live on the device; 4 % slack for imbalance) and
    // each group is then cut into equal tiles of at most that height on the device.
    int max_rows = 256;
    {
        const int tiles_n = (a.N + (sw ? 127 : 255)) / (sw ? 128 : 256);
        const int groups = a.group_offsets ? (a.n_groups > 0 ? a.n_groups : 1) : 1;
        const int r = !a.group_offsets ? rows
                      : a.m_expected > 0 ? (int)((int64_t)a.m_expected * 26 / 25) + 1
                                         : (int)((int64_t)rows * 26 / (25 * groups)) + 1;
        double best = 0;
        for (int cand = 256; cand >= 96; cand -= 32) {
            int nt, rt;
            split_rows(r, cand, nt, rt);
            const int jobs = groups * nt * tiles_n;
            const double cost = (double)((jobs + 255) / 256) * ((rt + 31) / 32 + 3);
            if (best == 0 || cost < best - 1e-9) { best = cost; max_rows = cand; }
        }
    }
    int wn_t = 4;
    {
        // a launch that gives at most half the compute units a 256-column tile (one expert of a small batch,
        // a short projection) is bound by how many units pull weights from HBM: halve the tile width
        int nt, rt;
        split_rows(a.group_offsets ? (a.m_expected > 0 ? a.m_expected : rows / (a.n_groups > 0 ? a.n_groups : 1)) : rows,
                   max_rows, nt, rt);
        const int64_t tiles = (int64_t)(a.group_offsets ? a.n_groups : 1) * nt * ((a.N + (sw ? 127 : 255)) / (sw ? 128 : 256));
        if (tiles <= 128 && a.epilogue != EPI_ROPE_KV) wn_t = 2;
    }
    if (a.force_max_rows > 0) max_rows = a.force_max_rows;
    if (a.force_wn_t == 2 || a.force_wn_t == 4) wn_t = a.force_wn_t;
    if (wn_t == 4) return sw ? launch_cfg<4, true>(a, max_rows, st) : launch_cfg<4, false>(a, max_rows, st);
    return sw ? launch_cfg<2, true>(a, max_rows, st) : launch_cfg<2, false>(a, max_rows, st);
}

}  // namespace sv
