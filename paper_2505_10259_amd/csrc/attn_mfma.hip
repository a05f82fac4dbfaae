// Paged-KV attention for the verify / draft / prefill passes on gfx950 (bf16, head_dim 128).
//
// One workgroup of two wavefronts per (sequence, KV head, block of 64 query rows); two workgroups share a
// compute unit (64 KB of LDS each, one wavefront per SIMD: the kernel holds about 350 registers).  The
// n_new query tokens times the g = Hq/Hkv query heads that share the KV head form n_new * g query rows;
// a verify or draft pass has at most 64 of them (one block), so every key/value byte read from HBM is
// used by all of them (the kernel is then HBM-bound: 4 KB of K+V per position per layer).  A prefill
// chunk of up to 64 prompt positions has up to 64 g rows: its row blocks run as separate workgroups
// (blockIdx.y), each over the keys its own rows may see (causal), re-reading the sequence's keys from L2.
//
//   * keys are processed in tiles of 32; wavefront w takes tiles w, w+2, ... with its own online
//     softmax state; the partial results are merged through LDS at the end;
//   * S^T = K Q^T and O^T = V^T P^T on v_mfma_f32_32x32x16_bf16, so that each lane owns one query
//     row (accumulator column): the softmax statistics are per-lane scalars and P goes from the
//     accumulator layout of the first product to the B-operand layout of the second without
//     leaving the lane; the Q fragments stay in registers for the whole loop;
//   * keys are row-major in a page and values are stored transposed ([dim][slot]), so both MFMA
//     operands are 16-byte pieces of memory rows; the key rows are fed in a fixed permutation (bits 2
//     and 3 of the row index swapped), which makes the 8 accumulator registers a lane converts to P
//     belong to 8 consecutive positions.  A tile travels HBM -> LDS with global_load_lds_dwordx4 in
//     1 KB runs (coalesced: measured, lane-private 16-byte gathers straight into registers kept the
//     vector cache busy with 64 lines per instruction and held the kernel at half the HBM rate) into
//     a per-wavefront ring of two 16 KB slots, and each lane reads its fragments back with
//     conflict-free swizzled ds_read_b128.  The ring is private to the wavefront: no barriers, and
//     two tiles per wavefront (128 KB per compute unit) are in flight while a third is multiplied;
//   * the softmax reference point of a row is only moved when the running maximum has grown by more
//     than 2^8 (the result does not depend on the reference; P stays below 2^8), so the rescaling of
//     the 128-wide output accumulator — by far the most expensive VALU work — is skipped for almost
//     every tile; the causal mask is applied only to tiles that reach the new tokens;
//   * the tile loads are issued from inline assembly (the compiler does not count them: the loop waits
//     with explicit vmcnt values), spread between the MFMAs of the tile being multiplied, and carry the
//     non-temporal hint when no other workgroup reads the same keys.
//
// What bounds it (MI355X, 256 sequences x 8 KV heads x 2057 positions, 36 query rows, 2.15 GB of K+V):
// a load-only copy of the request stream (same ring, no arithmetic) takes 0.353 ms without the hint and
// 0.318 ms with it (6.96 TB/s; a plain streaming read reaches 7.0-7.3 TB/s); this kernel with its
// arithmetic removed takes 0.337 ms, with its loads removed 0.208 ms, complete 0.373 ms (5.76 TB/s).
// Against the first version (four wavefronts, one workgroup per compute unit, 0.44 ms) the hint gave
// 0.023 ms, two-wavefront workgroups 0.011 ms (start-up and merge of one overlap the other's stream; 65
// tiles split 33/32 instead of 17/16), loads between the MFMAs 0.026 ms (sixteen loads issued back to
// back cost each wavefront about 1100 cycles per tile: the four wavefronts met in the address unit);
// earlier requests at start-up, one-barrier merge, Q in registers, and reading a tile's fragments half a
// step ahead into a second register set changed nothing measurable.
#include "common.h"
#include <type_traits>

namespace sv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

namespace {

constexpr int DH = 128;
constexpr float REF_SLACK = 8.0f;  // log2 units a row maximum may exceed its softmax reference
constexpr int TILE_BYTES = 16384;  // one 32-key tile: 8 KB of keys + 8 KB of values
constexpr int NW = 2;              // wavefronts per workgroup
constexpr int RING_BYTES = NW * 2 * TILE_BYTES;
constexpr int MAX_PAGES = 2048;    // page-table row kept in LDS (8 KB at most)

// eight accumulator values -> bf16 (round to nearest even; v_cvt_pk_bf16_f32 on gfx950)
__device__ inline bf16x8_t pack8(const f32x16_t& v, int base) {
    f32x8_t t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = v[base + i];
    return __builtin_convertvector(t, bf16x8_t);
}

// x of this lane and x of lane ^ 32, through v_permlane32_swap (register-file speed; a shuffle by 32
// would go through the LDS crossbar and cost a round trip per call)
__device__ inline void both_halves(float x, float& lo, float& hi) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    lo = __uint_as_float(r[0]);
    hi = __uint_as_float(r[1]);
}

template <int CT, bool NT>
__global__ void __launch_bounds__(64 * NW)
attn_mfma_kernel(AttnArgs a) {
    constexpr int RP = 32 * CT;
    // dynamic LDS: [ring: NW wavefronts x 2 slots x 16 KB | page-table row]; a wavefront's
    // partial output (RP rows x 128 floats) goes over its own ring slots once it has left its loop.  The page-table row is copied to
    // LDS once: a lookup in global memory inside the loop would have to wait on the vector-memory
    // counter, i.e. on every tile request still in flight.
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    __shared__ float sm_m[NW][RP], sm_l[NW][RP];
    int32_t* pts = (int32_t*)(smem + RING_BYTES);
    static_assert(RP * DH * 4 <= 2 * TILE_BYTES, "a partial output must fit in the wavefront's two ring slots");

    const int Hkv = a.geom.n_kv_heads;
    const int b = blockIdx.x / Hkv, kvh = blockIdx.x % Hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, hi = lane >> 5;
    const int g = a.n_q_heads / Hkv;
    const int row0 = (int)blockIdx.y * 64;                        // first query row of this workgroup's block
    const int rows = min(a.n_new * g - row0, 64);                 // rows of the block
    const int tok0 = row0 / g, tok1 = (row0 + rows - 1) / g;      // new tokens the block's rows belong to
    const bf16* kv = (const bf16*)a.kv_layer;
    const int ptok = a.geom.page_tokens;

    // The workgroup's first dependent memory step is page table -> tile address.  The pages of the tiles
    // this wavefront requests first (w and w+NW) are fetched together with the row positions, before the
    // number of tiles is known, so that start-up costs two memory latencies (these scalars, then the tiles;
    // the query rows and the page-table copy travel with the tiles).
    const int pps = a.geom.pages_per_seq;
    const int32_t* ptab = a.page_table + b * pps;
    const int sub_shift = __builtin_ctz((unsigned)(ptok >> 5)), sub_mask = (ptok >> 5) - 1;
    const int pg_a = ptab[min(w >> sub_shift, pps - 1)], pg_b = ptab[min((w + NW) >> sub_shift, pps - 1)];

    // keys [0, n_keys) exist; keys below mask_from are visible to every row of this workgroup
    int n_keys = 0, mask_from = 0x7fffffff;
    for (int i = tok0; i <= tok1; ++i) {
        int p = a.row_pos[b * a.n_new + i];
        n_keys = max(n_keys, p + 1);
        mask_from = min(mask_from, p < 0 ? 0 : p + 1);
    }
    const int n_tiles = (n_keys + 31) >> 5;
    const float c2 = a.scale * 1.4426950408889634f;      // scores in log2 units: exp2(s*c2 - m)

    int rpos[CT];
    bf16x8_t qf[CT][8];
    f32x16_t ot[4][CT];
    float m[CT], l[CT];          // m: softmax reference of the row (log2 units), l: sum of P
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        m[ct] = -INFINITY; l[ct] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) ot[dt][ct][r] = 0.f;
    }

    const int kperm = (c & ~12) | ((c & 8) >> 1) | ((c & 4) << 1);   // key row fed by this lane

    // Request tile `tile` into ring slot `slot` of this wavefront.  A tile is one 32-token sub-block of
    // a page: 16 KB of contiguous HBM, and every load instruction covers 1 KB of it (K: four 256-byte
    // key rows, V: sixteen 64-byte value rows), 8 cache lines per instruction; a direct-to-LDS load
    // puts lane i's 16 bytes at offset 16 i, so the LDS image is [row][16 chunks] for K and
    // [dim][4 chunks] for V.  Fragment reads take one 16-byte chunk per lane with 16 lanes (one LDS
    // cycle) on 16 different rows; the chunk order inside a row is therefore XOR-swizzled with the
    // row index (K: row & 15, V: (dim >> 2) & 3), applied here by choosing which global chunk a lane
    // fetches, which makes those reads conflict-free.
    //
    // A lane's byte offset inside the tile is the same for every tile, so it is computed once (16
    // registers) and a request is a scalar tile base plus that offset: the loop spends no vector
    // arithmetic on addresses (computed per request they were a third of the loop's instructions).
    char* ring = smem + w * 2 * TILE_BYTES;
    const int64_t page_stride = (int64_t)Hkv * 2 * ptok * DH * 2;              // bytes between pages
    const char* head_base = (const char*)kv + (int64_t)kvh * 2 * ptok * DH * 2;  // this head's block of page 0
    uint32_t koffs[8], voffs[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int r = 4 * q + (lane >> 4);
        koffs[q] = (uint32_t)(r * 256 + (((lane & 15) ^ (r & 15)) << 4));
        const int dim = 16 * q + (lane >> 2);
        voffs[q] = (uint32_t)(8192 + dim * 64 + (((lane & 3) ^ ((dim >> 2) & 3)) << 4));
    }
    // A request is split into its scalar part (tile -> 64-bit base address, LDS slot) and its sixteen load
    // instructions, issued from assembly with that scalar base and the lane's 32-bit offset.  The loop
    // issues them one at a time between the MFMAs of the tile it multiplies: issued back to back, the
    // wavefronts' requests met in the compute unit's address unit (16 cycles per 1 KB instruction) and
    // each wavefront sat about 1100 cycles per tile in the issue of its sixteen loads (measured with
    // s_memtime stamps), a quarter of its loop time, with nothing else to run on its SIMD.
    const uint32_t ring0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lds_ptr_t)ring);
    auto tile_base = [&](int64_t page, int tile) -> const char* {
        // page sizes are powers of two here (launcher), so tile -> (page, sub-block) is a shift and a mask
        return head_base + page * page_stride + (int64_t)(tile & sub_mask) * TILE_BYTES;   // wave-uniform
    };
    auto issue_load = [&](const char* tb, uint32_t dst, int q) {     // q in [0, 16): 8 key loads, 8 value loads
        const uint32_t d = dst + q * 1024;
        const uint32_t off = q < 8 ? koffs[q & 7] : voffs[q & 7];
        // NT: keys and values that no other workgroup reads again (one row block per KV head) are loaded
        // with the non-temporal hint; a load-only copy of this kernel's request stream ran at 6.27 TB/s
        // without the hint and 6.96 TB/s with it
        if (NT) asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" :: "s"(d), "v"(off), "s"(tb) : "memory", "m0");
        else asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(d), "v"(off), "s"(tb) : "memory", "m0");
    };
    auto request_tile = [&](const char* tb, int slot) {
        const uint32_t dst = ring0 + slot * TILE_BYTES;
#pragma unroll
        for (int q = 0; q < 16; ++q) issue_load(tb, dst, q);
    };
    // this lane's fragments: K row kperm, chunks 8 hi + kk; V dims dt*32 + c, chunks 2 t + hi
    // (the LDS offsets of these reads are per-lane constants as well)
    uint32_t kfo[8], vfo[4][2];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kfo[kk] = (uint32_t)(kperm * 256 + (((hi * 8 + kk) ^ (kperm & 15)) << 4));
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int dim = dt * 32 + c;
            vfo[dt][t] = (uint32_t)(8192 + dim * 64 + (((2 * t + hi) ^ ((dim >> 2) & 3)) << 4));
        }
    auto fetch_tile = [&](int slot, bf16x8_t (&kf)[8], bf16x8_t (&vf)[4][2]) {
        const char* src = ring + slot * TILE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) kf[kk] = *(const bf16x8_t*)(src + kfo[kk]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int t = 0; t < 2; ++t) vf[dt][t] = *(const bf16x8_t*)(src + vfo[dt][t]);
    };

    // (tb, dst): the tile requested while this one is multiplied; its 16 loads go out one per MFMA
    // (CT = 1) or one per two MFMAs (CT = 2)
    // (req = false: the last two tiles of a wavefront, nothing left to request)
    auto compute = [&](auto req, int tile, const bf16x8_t (&kf)[8], const bf16x8_t (&vf)[4][2], const char* tb, uint32_t dst) {
        constexpr bool REQ = decltype(req)::value;
        // the 16 loads are spread evenly over the tile's MFMAs (MFMA g = 16 ct + position in the column tile;
        // bunching them after the first MFMA or the first eight measured the same)
        constexpr int SPREAD = 16 * CT;
        auto loads_after = [&](int g) {
            const int lo = min(16, g * 16 / SPREAD), hi2 = min(16, (g + 1) * 16 / SPREAD);
#pragma unroll
            for (int q = lo; q < hi2; ++q) issue_load(tb, dst, q);
        };
        const int key0 = tile << 5;
        const bool need_mask = key0 + 32 > mask_from;          // wave-uniform
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            f32x16_t s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[ct][kk], s, 0, 0, 0);
                if (REQ) loads_after(ct * 16 + kk);
            }
            // register r of this lane <-> position key0 + 16*(r/8) + 8*hi + r%8
            if (need_mask) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int kp = key0 + ((r >> 3) << 4) + (hi << 3) + (r & 7);
                    s[r] = kp <= rpos[ct] ? s[r] : -INFINITY;
                }
            }
            // the scale (positive) is applied to the maximum and, fused with the subtraction of the
            // reference, inside the exponent: one FMA per score instead of a multiply and a subtract
            float mx = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
            {
                float x0, x1;
                both_halves(mx, x0, x1);
                mx = fmaxf(x0, x1) * c2;
            }
            // move the reference only when the maximum outgrew it by more than the slack
            const bool upd = mx > m[ct] + REF_SLACK;            // m = -inf: any finite mx updates
            const float m_new = upd ? mx : m[ct];
            const float mref = m_new == -INFINITY ? 0.f : m_new;   // row has seen nothing: p = 0
            const float corr = upd ? __builtin_amdgcn_exp2f(m[ct] - mref) : 1.f;
            float ps = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c2, -mref)); s[r] = p; ps += p; }
            {
                float x0, x1;
                both_halves(ps, x0, x1);
                ps = x0 + x1;
            }
            l[ct] = l[ct] * corr + ps;
            m[ct] = m_new;
            if (__any(upd)) {                                    // wave-uniform; corr = 1 elsewhere
                // rare (the reference moves only when the maximum outgrows it by the slack).  Written as
                // assembly on the accumulator registers so that their 64 reads stay inside this branch:
                // as plain multiplies the compiler hoisted the reads out and paid them for every tile.
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float t;
                        asm volatile("v_accvgpr_read_b32 %1, %0\n\ts_nop 0\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n\t"
                                     "v_accvgpr_write_b32 %0, %1"
                                     : "+a"(ot[dt][ct][r]), "=&v"(t) : "v"(corr));
                    }
            }
            bf16x8_t p0 = pack8(s, 0), p1 = pack8(s, 8);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                ot[dt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][0], p0, ot[dt][ct], 0, 0, 0);
                if (REQ) loads_after(ct * 16 + 8 + 2 * dt);
                ot[dt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][1], p1, ot[dt][ct], 0, 0, 0);
                if (REQ) loads_after(ct * 16 + 9 + 2 * dt);
            }
        }
    };

    // ---- query rows of this lane (one per column tile) --------------------------------------------
    // Every wavefront keeps all Q fragments in registers for its whole loop (64 registers for two column
    // tiles; one wavefront per SIMD has 512) and loads them straight from global memory in fragment
    // layout: lane (c, hi) takes the 128 bytes [hi*64, hi*64+64) of query row ct*32 + c.  These loads and
    // the page-table row are issued first and the wavefront's first two tiles right behind them.
    // (unconditional loads from clamped addresses: a load under a branch makes the compiler wait for it
    // at the end of the branch)
    const int pt_mine = ptab[min(tid, pps - 1)];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int rr = min(ct * 32 + c, rows - 1);
        const int i = (row0 + rr) / g, j = (row0 + rr) % g;
        const int t = b * a.n_new + i;
        rpos[ct] = a.row_pos[t];
        const bf16* qp = (const bf16*)a.q + ((int64_t)t * a.n_q_heads + kvh * g + j) * DH + hi * 64;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[ct][kk] = *(const bf16x8_t*)(qp + kk * 8);
    }
    const int my_tiles = w < n_tiles ? (n_tiles - w + NW - 1) / NW : 0;     // tiles w, w+NW, ... of this wavefront
    if (my_tiles > 0) request_tile(tile_base(__builtin_amdgcn_readfirstlane(pg_a), w), 0);
    if (my_tiles > 1) request_tile(tile_base(__builtin_amdgcn_readfirstlane(pg_b), w + NW), 1);
    if (tid < pps) pts[tid] = pt_mine;
    for (int i = tid + 64 * NW; i < pps; i += 64 * NW) pts[i] = ptab[i];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const bool valid = ct * 32 + c < rows;           // rows past the block: zero query, nothing visible
        if (!valid) rpos[ct] = -1;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[ct][kk][e] = valid ? qf[ct][kk][e] : (__bf16)0.0f;
    }
    __syncthreads();

    if (my_tiles > 0) {
        // Iteration i multiplies tile w + NW i from registers while tiles i+1 and i+2 are on their way
        // into the two ring slots.  Loads complete in issue order, so "at most 16 outstanding" means
        // that everything but the newest tile has landed.  The inline-asm waits also keep the
        // compiler from moving the LDS reads across them.  The last two iterations have nothing left
        // to request and wait for everything.
        bf16x8_t kf[8], vf[4][2];
        if (my_tiles > 1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        fetch_tile(0, kf, vf);
        int tile = w, i = 0;
        for (; i < my_tiles - 2; ++i) {
            const int nt = tile + 2 * NW;
            const char* tb = tile_base(__builtin_amdgcn_readfirstlane(pts[nt >> sub_shift]), nt);
            // the fragments of tile i have reached the registers: its slot can be overwritten
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            compute(std::true_type{}, tile, kf, vf, tb, ring0 + (i & 1) * TILE_BYTES);
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            fetch_tile((i + 1) & 1, kf, vf);
            tile += NW;
        }
        for (; i < my_tiles; ++i) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            compute(std::false_type{}, tile, kf, vf, nullptr, 0u);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (i + 1 < my_tiles) fetch_tile((i + 1) & 1, kf, vf);
            tile += NW;
        }
    }
    // ---- merge the wavefronts' partial softmaxes --------------------------------------------
    // A wavefront that has left its loop (all its requests have landed and been read) puts its
    // un-normalised partial output over its own two ring slots, 512 bytes per query row, and its (m, l)
    // per row beside it: no barrier before that, so wavefronts with fewer tiles do this while the
    // others still multiply.  The 16-byte chunks of a row are XOR-swizzled with the row index, which
    // keeps both the writes here (16 lanes on 16 rows) and the row-wise reads below conflict-free.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    {
        float* mine = (float*)ring;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const int row = ct * 32 + c;
            if (hi == 0) { sm_m[w][row] = m[ct]; sm_l[w][row] = l[ct]; }
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    // registers 4q..4q+3 <-> dims dt*32 + 8q + 4*hi + 0..3 of query row ct*32+c
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = ot[dt][ct][4 * q + e];
                    const int chunk = dt * 8 + 2 * q + hi;
                    *(f32x4_t*)(mine + row * DH + ((chunk ^ (row & 15)) << 2)) = v;
                }
        }
    }
    __syncthreads();
    // ---- write out: wavefront w takes rows w, w+NW, ...; a lane two adjacent dims (coalesced).  The
    // partials are brought to the common reference M = max m_w and added: out = sum_w f_w O_w / sum_w f_w l_w
#pragma unroll 3
    for (int rr = w; rr < rows; rr += NW) {
        const int i = (row0 + rr) / g, j = (row0 + rr) % g;
        float mw[NW], f[NW];
        float M = -INFINITY;
#pragma unroll
        for (int q = 0; q < NW; ++q) { mw[q] = sm_m[q][rr]; M = fmaxf(M, mw[q]); }
        float L = 0.f, x0 = 0.f, x1 = 0.f;
#pragma unroll
        for (int q = 0; q < NW; ++q) {
            f[q] = mw[q] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw[q] - M);
            L += sm_l[q][rr] * f[q];
            const float2 v = *(const float2*)(smem + q * 2 * TILE_BYTES + rr * (DH * 4) +
                                              ((((lane >> 1) ^ (rr & 15)) << 4) | ((lane & 1) << 3)));
            x0 += v.x * f[q]; x1 += v.y * f[q];
        }
        const float inv = L > 0.f ? 1.0f / L : 0.f;
        bf16* op = (bf16*)a.out + ((int64_t)(b * a.n_new + i) * a.n_q_heads + kvh * g + j) * DH + 2 * lane;
        uint32_t lo = f32_to_bf16(x0 * inv).bits;
        uint32_t hi16 = f32_to_bf16(x1 * inv).bits;
        *(uint32_t*)op = lo | (hi16 << 16);
    }
}

}  // namespace

hipError_t launch_attention_mfma_bf16(const AttnArgs& a, hipStream_t st) {
    if (a.B <= 0 || a.n_new <= 0) return hipSuccess;
    int g = a.n_q_heads / a.geom.n_kv_heads;
    int rows = a.n_new * g;
    // the MFMA kernel covers the shapes of the supported models; anything else takes the plain one
    // (pages of 32, 64, 128, ... tokens: the kernel turns a tile index into page and sub-block by shifting)
    const int pt = a.geom.page_tokens;
    if (a.geom.head_dim != DH || pt < 32 || (pt & (pt - 1)) != 0 || a.geom.pages_per_seq > MAX_PAGES)
        return launch_attention_simple(a, SPEC_BF16, st);
    dim3 grid(a.B * a.geom.n_kv_heads, (rows + 63) / 64);
    static bool attr_set = false;
    if (!attr_set) {
        const void* fns[4] = {(const void*)attn_mfma_kernel<1, false>, (const void*)attn_mfma_kernel<1, true>,
                              (const void*)attn_mfma_kernel<2, false>, (const void*)attn_mfma_kernel<2, true>};
        for (int i = 0; i < 4; ++i) {
            hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize,
                                               RING_BYTES + MAX_PAGES * 4);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    const int pt_bytes = a.geom.pages_per_seq * 4;
    const int ct = rows <= 32 ? 1 : 2;
    const size_t lds = RING_BYTES + pt_bytes;
    const bool nt = grid.y == 1;          // several row blocks share the keys through L2: no hint there
    if (ct == 1 && nt) hipLaunchKernelGGL((attn_mfma_kernel<1, true>), grid, dim3(64 * NW), lds, st, a);
    else if (ct == 1) hipLaunchKernelGGL((attn_mfma_kernel<1, false>), grid, dim3(64 * NW), lds, st, a);
    else if (nt) hipLaunchKernelGGL((attn_mfma_kernel<2, true>), grid, dim3(64 * NW), lds, st, a);
    else hipLaunchKernelGGL((attn_mfma_kernel<2, false>), grid, dim3(64 * NW), lds, st, a);
    return hipGetLastError();
}

}  // namespace sv
