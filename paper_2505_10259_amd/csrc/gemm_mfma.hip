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
//     weights three slabs deep and the activations two (three where 160 KB allow), one barrier per
//     slab; the loads are issued from inline assembly, one per accumulator row of MFMAs, and waited
//     for with a counted vmcnt (see the pipeline comment in gemm_tile for why and what was measured);
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

    // ---- per-lane global source addresses of this lane's 16-byte chunks ------------------------
    const int lrow = lane >> 3;                 // row inside an 8-row load group
    // swizzle key of tile row r is (r >> 1) & 7; load group q covers rows 8q..8q+7, so a lane's key
    // is (4q + lane/16) & 7 and it fetches global chunk (lane & 7) ^ key into slot lane & 7
    auto gchunk_of = [&](int q) { return (lane & 7) ^ ((4 * q + (lane >> 4)) & 7); };
    // (per-lane 64-bit addresses, advanced by the slab with two VALU adds per load: the scalar-base +
    // 32-bit-offset form of the same loads measured 17 % slower on the grouped MoE product)
    const char* a_src[A_INST];
    const char* b_src[B_INST];
#pragma unroll
    for (int j = 0; j < A_INST; ++j) {
        int r = row_begin + (w * A_INST + j) * 8 + lrow;
        r = r < row_end ? r : row_end - 1;                       // clamp: masked at the store
        int64_t src = a.a_rows ? (int64_t)a.a_rows[r] : (int64_t)r;
        a_src[j] = Ab + (src * a.lda + gchunk_of(w * A_INST + j) * 8) * 2;
    }
#pragma unroll
    for (int j = 0; j < B_INST; ++j) {
        int tr = (w * B_INST + j) * 8 + lrow;                   // row of the B tile, 0..BN-1
        const char* base = Wb;
        int n;
        if (SWIGLU) {
            // a wavefront column block = [its gate features | the same up features]
            int wcol = tr / (BN / 2), within = tr % (BN / 2);
            bool up = within >= BN / 4;
            n = n0 + wcol * (BN / 4) + (up ? within - BN / 4 : within);
            base = up ? W3b : Wb;
        } else {
            n = n0 + tr;
        }
        n = n < a.N ? n : a.N - 1;
        b_src[j] = base + ((int64_t)n * a.K + gchunk_of(w * B_INST + j) * 8) * 2;
    }

    // Direct-to-LDS loads are issued from inline assembly: to the compiler's wait-count pass a pending
    // LDS-DMA load forces every later wait for a fragment read to drain all reads (lgkmcnt(0)), which
    // stalls a wavefront for the whole read queue each time a load sits between two MFMAs; hidden from
    // it, fragment waits are counted, and the loads' own completion is waited for by hand (vmcnt) at the
    // head of a slab.  The LDS destination of lane i is M0 + 16 i.
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lds_ptr_t)smem);
    const uint32_t wu = (uint32_t)w;
    auto issue_a = [&](int q, int kt, int ast) {     // load q of activation slab kt into A stage ast
        const uint32_t dst = lds0 + ast * A_BYTES + (wu * A_INST + q) * 1024;
        const char* src = a_src[q] + (int64_t)kt * 128;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(dst), "v"(src) : "memory", "m0");
    };
    auto issue_b = [&](int q, int kt, int bst) {     // load q of weight slab kt into B stage bst
        const uint32_t dst = lds0 + B_BASE + bst * B_BYTES + (wu * B_INST + q) * 1024;
        const char* src = b_src[q] + (int64_t)kt * 128;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(dst), "v"(src) : "memory", "m0");
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

    // Pipeline.  Weight slabs are three deep in LDS, activation slabs two (three where they fit): the
    // weights of a grouped product mostly come from HBM (each is used by the few row tiles of one expert)
    // and need about two slab times to arrive, the activations are re-read by every column tile and hit
    // in L2.  In slab kt a wavefront issues the loads of A(kt+1), then of B(kt+2), ONE in front of each accumulator row of
    // MFMAs (8 MFMAs): spread like this the requests of a compute unit do not queue behind each other
    // (issued as one burst at the head of the slab the same kernel measured 957 instead of 1037 TFLOP/s
    // on the MoE product).  Loads complete in issue order, so the head of slab kt waits until at most the
    // B(kt+1) loads are pending (vmcnt(B_INST)): A(kt) and B(kt) have landed; the barrier then also says
    // that every wavefront has finished reading slab kt-1, whose A stage and B stage the new loads
    // overwrite.  Fragment reads of both k-steps are issued at the head of the slab; the compiler waits
    // for them with counted lgkmcnt.  sched_barrier pins the load positions (MFMAs are otherwise free
    // to move across the assembly statements).
    auto slab = [&](int kt, int bst, auto mode_c, auto wait_c) {
        // MODE 2: issue A(kt+1) (A(kt+2) when the activations are three deep) and B(kt+2); 1: A(kt+1); 0: none
        constexpr int MODE = decltype(mode_c)::value;
        constexpr int WAITN = decltype(wait_c)::value;           // loads that may stay pending
        __builtin_amdgcn_s_waitcnt(0x0F70 | WAITN);              // vmcnt(WAITN)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const char* As = smem + (AST == 3 ? bst : kt & 1) * A_BYTES;
        const char* Bs = smem + B_BASE + bst * B_BYTES;
        const int bst2 = bst == 0 ? 2 : bst - 1;                 // (bst + 2) % 3
        bf16x8_t af[2][MI], bfr[2][NI];
        auto load_frags = [&](int kk) {
            const int coff = ((4 * kk + kquart) ^ sw) << 4;
#pragma unroll
            for (int i = 0; i < MI; ++i) af[kk][i] = *(const bf16x8_t*)(As + a_off + i * 16 * 128 + coff);
#pragma unroll
            for (int j = 0; j < NI; ++j) bfr[kk][j] = *(const bf16x8_t*)(Bs + b_off + j * 16 * 128 + coff);
        };
        auto issue_seq = [&](int v) {        // A loads first: the wait of the next slab leaves the B loads pending
            if (v < A_INST) {
                if (AST == 3) { if (MODE >= 2) issue_a(v, kt + 2, bst2); }
                else if (MODE >= 1) issue_a(v, kt + 1, (kt + 1) & 1);
            } else if (MODE >= 2) issue_b(v - A_INST, kt + 2, bst2);
        };
        load_frags(0);
        load_frags(1);
#pragma unroll
        for (int r = 0; r < 2 * MI; ++r) {
            const int kk = r / MI, i = r % MI;
            if (r < NL) issue_seq(r);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[kk][j], af[kk][i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int v = 2 * MI; v < NL; ++v) issue_seq(v);           // short tiles: the rest in one go
    };

    const int KT = a.K / 64;
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    // loads that may be pending at the head of a slab: those of the next slab that were issued a slab early
    using IB = std::integral_constant<int, AST == 3 ? NL : B_INST>;
#pragma unroll
    for (int q = 0; q < A_INST; ++q) issue_a(q, 0, 0);
#pragma unroll
    for (int q = 0; q < B_INST; ++q) issue_b(q, 0, 0);
    if (KT == 1) {
        slab(0, 0, I0{}, I0{});
    } else {
        if (AST == 3) {
#pragma unroll
            for (int q = 0; q < A_INST; ++q) issue_a(q, 1, 1);
        }
#pragma unroll
        for (int q = 0; q < B_INST; ++q) issue_b(q, 1, 1);
        int bst = 0;
        for (int kt = 0; kt + 2 < KT; ++kt) { slab(kt, bst, I2{}, IB{}); bst = bst == 2 ? 0 : bst + 1; }
        slab(KT - 2, bst, I1{}, IB{});
        slab(KT - 1, bst == 2 ? 0 : bst + 1, I0{}, I0{});
    }

    // ---- epilogue: tile (i, j) of a lane: output row i*16 + (lane & 15), columns j*16 + 4*(lane/16)
    // + 0..3 (the weight fragment was the A operand), stored as one 16- or 8-byte vector; the launcher
    // guarantees N and the row pitch are multiples of 4.
    const int row_in = lane & 15, cq = (lane >> 4) * 4;
    if constexpr (SWIGLU) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int row = row_begin + wm * 16 * MI + i * 16 + row_in;
#pragma unroll
            for (int j = 0; j < NI / 2; ++j) {
                const int col = n0 + wn * (BN / 4) + j * 16 + cq;
                f32x4_t g = acc[i][j], u = acc[i][j + NI / 2], p;
#pragma unroll
                for (int r = 0; r < 4; ++r) p[r] = g[r] / (1.0f + __expf(-g[r])) * u[r];
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
                    f32x4_t lo[4], hi[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) { lo[j] = acc[i][j]; hi[j] = acc[i][j + 4]; }
                    if (head < Hq + Hkv) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float2* cp = rp.cs + (int64_t)row * 64 + j * 16 + cq;
                            const f32x4_t c01 = *(const f32x4_t*)cp, c23 = *(const f32x4_t*)(cp + 2);
                            const float cs_c[4] = {c01[0], c01[2], c23[0], c23[2]};
                            const float cs_s[4] = {c01[1], c01[3], c23[1], c23[3]};
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float x0 = lo[j][r], x1 = hi[j][r];
                                lo[j][r] = x0 * cs_c[r] - x1 * cs_s[r];
                                hi[j][r] = x1 * cs_c[r] + x0 * cs_s[r];
                            }
                        }
                    }
                    if (head < Hq) {
                        bf16* dst = (bf16*)rp.q_out + ((int64_t)row * Hq + head) * 128;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            *(bf16x4_t*)(dst + j * 16 + cq) = __builtin_convertvector(lo[j], bf16x4_t);
                            *(bf16x4_t*)(dst + 64 + j * 16 + cq) = __builtin_convertvector(hi[j], bf16x4_t);
                        }
                        continue;
                    }
                    const int pos = rp.row_pos[row];
                    if (pos < 0) continue;
                    const int lp = pos / rp.geom.page_tokens;
                    if (lp >= rp.geom.pages_per_seq) continue;
                    const int64_t page = rp.page_table[(row / rp.n_new) * rp.geom.pages_per_seq + lp];
                    const int slot = pos % rp.geom.page_tokens;
                    bf16* kvp = (bf16*)rp.kv_layer;
                    if (head < Hq + Hkv) {
                        bf16* dst = kvp + rp.geom.k_off(page, head - Hq, slot);
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            *(bf16x4_t*)(dst + j * 16 + cq) = __builtin_convertvector(lo[j], bf16x4_t);
                            *(bf16x4_t*)(dst + 64 + j * 16 + cq) = __builtin_convertvector(hi[j], bf16x4_t);
                        }
                    } else {
                        const int kvh = head - Hq - Hkv;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                kvp[rp.geom.v_off(page, kvh, slot, j * 16 + cq + r)] = f32_to_bf16(lo[j][r]);
                                kvp[rp.geom.v_off(page, kvh, slot, 64 + j * 16 + cq + r)] = f32_to_bf16(hi[j][r]);
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

template <int WN_T, bool SWIGLU>
__global__ void __launch_bounds__(256, 1)
gemm_bf16_mfma_kernel(GemmArgs a, int max_rows, int tiles_n) {
    constexpr int BN = 64 * WN_T;
    constexpr int N_OUT = SWIGLU ? BN / 2 : BN;       // output columns per workgroup
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // ---- which tile: workgroup id x runs on XCD x % 8, and each XCD takes one contiguous range of the
    // logical tile order (see the head of this file)
    int total = 0;
    if (a.group_offsets) {
        for (int g = 0; g < a.n_groups; ++g) {
            int nt, rt;
            split_rows(a.group_offsets[g + 1] - a.group_offsets[g], max_rows, nt, rt);
            total += nt * tiles_n;
        }
    } else {
        int nt, rt;
        split_rows(a.M, max_rows, nt, rt);
        total = nt * tiles_n;
    }
    const int per_xcd = (total + 7) >> 3;
    const int slot = (int)(blockIdx.x >> 3);
    const int logical = (int)(blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || logical >= total) return;
    int tile_m = 0, tile_n = 0, row_begin = 0, row_end = 0, group = 0;
    if (a.group_offsets) {
        int base = 0;
        for (int g = 0; g < a.n_groups; ++g) {
            const int b0 = a.group_offsets[g], b1 = a.group_offsets[g + 1];
            int nt, rt;
            split_rows(b1 - b0, max_rows, nt, rt);
            const int local = logical - base;
            if (local >= 0 && local < nt * tiles_n) {
                group = g;
                band_order(local, nt, tiles_n, tile_m, tile_n);
                row_begin = b0 + tile_m * rt;
                row_end = row_begin + rt < b1 ? row_begin + rt : b1;
            }
            base += nt * tiles_n;
        }
    } else {
        int nt, rt;
        split_rows(a.M, max_rows, nt, rt);
        band_order(logical, nt, tiles_n, tile_m, tile_n);
        row_begin = tile_m * rt;
        row_end = row_begin + rt < a.M ? row_begin + rt : a.M;
    }
    const int rows = row_end - row_begin;
    if (rows <= 0) return;          // rounding the tile height up to 16 can leave a last tile empty
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
}

template <int WN_T, bool SWIGLU>
hipError_t launch_cfg(const GemmArgs& a, int max_rows, hipStream_t st) {
    constexpr int BN = 64 * WN_T;
    constexpr int N_OUT = SWIGLU ? BN / 2 : BN;
    constexpr int SMEM = (2 * 256 + 3 * BN) * 128;        // two activation stages of the tallest tile, three weight stages
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
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), SMEM, st, a, max_rows, tiles_n);
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
    if (wn_t == 4) return sw ? launch_cfg<4, true>(a, max_rows, st) : launch_cfg<4, false>(a, max_rows, st);
    return sw ? launch_cfg<2, true>(a, max_rows, st) : launch_cfg<2, false>(a, max_rows, st);
}

}  // namespace sv
