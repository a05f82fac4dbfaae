// bf16 MFMA GEMM for gfx950:  C[M,N] (+)= A[M,K] * W[N,K]^T, f32 accumulate, with
//   - optional row gather on A and row grouping with per-group weights (top-2 MoE grouped GEMM),
//   - fused epilogues: f32 store, f32 residual accumulate, bf16 store, SwiGLU (two weight
//     matrices, silu(gate) * up, bf16 store).
//
// Design (64-wide wavefronts, CDNA4):
//   * workgroup = 4 wavefronts in a 2x2 grid; each wavefront owns a (32*WM_T) x (32*WN_T) block of
//     v_mfma_f32_32x32x16_bf16 tiles held in accumulator registers;
//   * operands go global -> LDS with global_load_lds_dwordx4 (no VGPR staging), 64-wide K slabs,
//     double buffered; one barrier per slab;
//   * LDS rows are 128 B (64 bf16); the 16-byte chunk c of row r is stored at chunk position
//     c ^ (r & 7) so that the 8 rows read together by ds_read_b128 hit 8 different bank groups.
//     Direct-to-LDS loads place lane i at base + 16*i, so the swizzle is applied by choosing which
//     global chunk a lane fetches;
//   * tile order: row tiles fastest (neighbouring workgroups share the weight slab), and the linear
//     workgroup id is remapped so that each XCD (id % 8) walks one contiguous range of tiles, i.e.
//     every weight slab is pulled into exactly one XCD's L2.
#include "common.h"

namespace sv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

namespace {

template <int WM_T, int WN_T, bool SWIGLU>
__global__ void __launch_bounds__(256, 1)
gemm_bf16_mfma_kernel(GemmArgs a, int row_tiles_max, int total_tiles, int per_xcd) {
    constexpr int BM = 64 * WM_T, BN = 64 * WN_T;
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
    constexpr int N_OUT = SWIGLU ? BN / 2 : BN;       // output columns per workgroup
    constexpr int A_INST = BM / 32, B_INST = BN / 32; // direct-to-LDS loads per wavefront per slab
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
    if (logical >= total_tiles) return;
    const int tile_n = logical / row_tiles_max;
    int rt = logical % row_tiles_max;

    int row_begin, row_end, group = 0;
    if (a.group_offsets) {
        bool found = false;
        int acc_tiles = 0;
        row_begin = row_end = 0;
        for (int g = 0; g < a.n_groups; ++g) {
            int b0 = a.group_offsets[g], b1 = a.group_offsets[g + 1];
            int nt = (b1 - b0 + BM - 1) / BM;
            if (!found && rt < acc_tiles + nt) {
                group = g; row_begin = b0 + (rt - acc_tiles) * BM; row_end = b1; found = true;
            }
            acc_tiles += nt;
        }
        if (!found) return;
    } else {
        row_begin = rt * BM;
        row_end = a.M;
        if (row_begin >= row_end) return;
    }
    const int n0 = tile_n * N_OUT;

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int wm = w >> 1, wn = w & 1;
    const char* Ab = (const char*)a.A;
    const char* Wb = (const char*)a.W + (int64_t)group * a.w_group_stride * 2;
    const char* W3b = SWIGLU ? (const char*)a.W3 + (int64_t)group * a.w_group_stride * 2 : nullptr;

    // ---- per-lane global source addresses of this lane's 16-byte chunks ------------------------
    const int lrow = lane >> 3;                 // row inside an 8-row load group
    const int gchunk = (lane & 7) ^ lrow;       // swizzle: global chunk fetched into slot lane&7
    const char* a_src[A_INST];
    const char* b_src[B_INST];
#pragma unroll
    for (int j = 0; j < A_INST; ++j) {
        int r = row_begin + (w * A_INST + j) * 8 + lrow;
        r = r < row_end ? r : row_end - 1;                       // clamp: masked at the store
        int64_t src = a.a_rows ? (int64_t)a.a_rows[r] : (int64_t)r;
        a_src[j] = Ab + (src * a.lda + gchunk * 8) * 2;
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
        b_src[j] = base + ((int64_t)n * a.K + gchunk * 8) * 2;
    }

    auto issue = [&](int stage, int k0) {
        char* As = smem + stage * STAGE;
        char* Bs = As + A_BYTES;
#pragma unroll
        for (int j = 0; j < A_INST; ++j)
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(a_src[j] + (int64_t)k0 * 2),
                                             (lds_ptr_t)(As + (w * A_INST + j) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < B_INST; ++j)
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(b_src[j] + (int64_t)k0 * 2),
                                             (lds_ptr_t)(Bs + (w * B_INST + j) * 1024), 16, 0, 0);
    };

    f32x16_t acc[WM_T][WN_T];
#pragma unroll
    for (int i = 0; i < WM_T; ++i)
#pragma unroll
        for (int j = 0; j < WN_T; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment read offsets: row (lane & 31) of each 32-row tile, chunk (2*kk + lane/32) ^ (lane & 7)
    const int frag_row = lane & 31, khalf = lane >> 5, sw = lane & 7;
    const int a_off = (wm * 32 * WM_T + frag_row) * 128;
    const int b_off = (wn * 32 * WN_T + frag_row) * 128;

    const int KT = a.K / 64;
    issue(0, 0);
    for (int kt = 0; kt < KT; ++kt) {
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): this wavefront's slab loads landed
        __syncthreads();                             // ... and everyone else's; previous slab fully read
        if (kt + 1 < KT) issue((kt + 1) & 1, (kt + 1) * 64);
        const char* As = smem + (kt & 1) * STAGE;
        const char* Bs = As + A_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int coff = ((2 * kk + khalf) ^ sw) << 4;
            bf16x8_t af[WM_T], bfr[WN_T];
#pragma unroll
            for (int i = 0; i < WM_T; ++i) af[i] = *(const bf16x8_t*)(As + a_off + i * 32 * 128 + coff);
#pragma unroll
            for (int j = 0; j < WN_T; ++j) bfr[j] = *(const bf16x8_t*)(Bs + b_off + j * 32 * 128 + coff);
#pragma unroll
            for (int i = 0; i < WM_T; ++i)
#pragma unroll
                for (int j = 0; j < WN_T; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    }

    // ---- epilogue: lane holds column (lane & 31); register r -> row 8*(r/4) + 4*(lane/32) + r%4 ----
    const int col_in = lane & 31, rgrp = lane >> 5;
#pragma unroll
    for (int i = 0; i < WM_T; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int row = row_begin + wm * 32 * WM_T + i * 32 + 8 * (r >> 2) + 4 * rgrp + (r & 3);
            if (row >= row_end) continue;
            if (SWIGLU) {
#pragma unroll
                for (int j = 0; j < WN_T / 2; ++j) {
                    int col = n0 + wn * (BN / 4) + j * 32 + col_in;
                    if (col >= a.N) continue;
                    float g = acc[i][j][r], u = acc[i][j + WN_T / 2][r];
                    float s = g / (1.0f + __expf(-g));
                    ((bf16*)a.C)[(int64_t)row * a.ldc + col] = f32_to_bf16(s * u);
                }
            } else {
#pragma unroll
                for (int j = 0; j < WN_T; ++j) {
                    int col = n0 + wn * 32 * WN_T + j * 32 + col_in;
                    if (col >= a.N) continue;
                    int64_t o = (int64_t)row * a.ldc + col;
                    float v = acc[i][j][r];
                    if (a.epilogue == EPI_STORE_F32) ((float*)a.C)[o] = v;
                    else if (a.epilogue == EPI_ADD_F32) ((float*)a.C)[o] += v;
                    else ((bf16*)a.C)[o] = f32_to_bf16(v);
                }
            }
        }
    }
}

template <int WM_T, int WN_T, bool SWIGLU>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t st) {
    constexpr int BM = 64 * WM_T, BN = 64 * WN_T;
    constexpr int N_OUT = SWIGLU ? BN / 2 : BN;
    constexpr int SMEM = 2 * (BM + BN) * 128;
    static bool attr_set = false;
    auto kern = gemm_bf16_mfma_kernel<WM_T, WN_T, SWIGLU>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int rows = a.group_offsets ? a.m_upper : a.M;
    int row_tiles = (rows + BM - 1) / BM + (a.group_offsets ? a.n_groups : 0);
    int tiles_n = (a.N + N_OUT - 1) / N_OUT;
    int total = row_tiles * tiles_n;
    int per_xcd = (total + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(256), SMEM, st, a, row_tiles, total, per_xcd);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_mfma_bf16(const GemmArgs& a, hipStream_t st) {
    int rows = a.group_offsets ? a.m_upper : a.M;
    if (rows <= 0 || a.N <= 0) return hipSuccess;
    // the MFMA path needs whole 64-wide K slabs and 16-byte aligned rows; anything else (never the
    // case for the supported model shapes) takes the plain kernel
    if (a.K % 64 != 0 || a.lda % 8 != 0 || ((uintptr_t)a.A & 15) || ((uintptr_t)a.W & 15))
        return launch_gemm_simple(a, SPEC_BF16, st);
    const bool sw = a.epilogue == EPI_SWIGLU_T;
    // tile choice: big tiles when there are enough rows to fill them
    int avg_rows = a.group_offsets ? rows / (a.n_groups > 0 ? a.n_groups : 1) : rows;
    if (avg_rows > 128) {
        if (sw) return launch_cfg<4, 4, true>(a, st);
        return launch_cfg<4, 4, false>(a, st);
    }
    if (sw) return launch_cfg<2, 4, true>(a, st);
    return launch_cfg<2, 4, false>(a, st);
}

}  // namespace sv
