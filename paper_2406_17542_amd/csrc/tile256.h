// A 256 x 256 tile of C = A^T B on the matrix cores, for 16-bit operands stored contraction-major: A [k][m] and B [k][n] with
// rows of the contraction index k (the tokens of X for H = X^T X; the input coordinates for a product with the symmetric
// R).  One workgroup of 4 wavefronts (one per SIMD), each 128 x 128 = 4 x 4 blocks of a 32x32x16 MFMA with the 256
// accumulator registers in AGPRs.  Shared by the Hessian kernel and the OWC screen.
//
// The contraction is consumed in steps of 32 rows; LDS is a ring of NSTAGE stages, each holding the two operand tiles of
// one step as 32 rows of 256 elements (512 bytes).  A wavefront's direct global->LDS load moves 64 x 16 bytes = two rows;
// lane l writes chunk position l%32 of row l/32 and fetches the global 16-byte chunk (l%32) ^ 4(row%4), i.e. the chunks of
// a row are XOR-swizzled by the row.  A transposing read (ds_read_b64_tr_b16) by the 16 lanes j of a group fetches the
// 8-byte pieces (row rb + j/4, elements fb + 4(j%4) .. +3) and returns to lane j the rows rb .. rb+3 of element fb + j;
// with the swizzle the four rows of a group fall into four different 64-byte bank groups, so reads and writes are
// conflict-free.
// With a single wavefront per SIMD nothing else hides a stall, so the loop is a software pipeline over quarters of a
// 16-row half step: four MFMAs, the four LDS reads that fetch a quarter of the next half's fragments, and ONE of the
// wavefront's eight loads of a later step.  Issuing a step's loads in one burst held every wavefront in its issue
// sequence while the CU's single address unit worked through 32 KiB -- about 500 cycles per 1000-cycle step with the
// matrix cores idle; spread out, a load costs the wavefront a scalar add and a move.  Loads run NSTAGE-1 steps ahead; the
// one barrier per step sits between the two halves.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cdq {
namespace tile256 {

typedef float acc16 __attribute__((ext_vector_type(16)));
typedef short frag8 __attribute__((ext_vector_type(8)));       // 8 contraction elements of one row/column, as 16-bit patterns
typedef short s4v __attribute__((ext_vector_type(4)));

constexpr int T2 = 256;                 // tile edge
constexpr int BKS = 32;                 // contraction rows per step
constexpr int ROWB = T2 * 2;            // LDS bytes per row of an operand tile
constexpr int TILE_BYTES = BKS * ROWB;  // 16 KiB per operand per stage
constexpr int STAGE = 2 * TILE_BYTES;
constexpr int NSTAGE = 4;
constexpr int LDS_BYTES = NSTAGE * STAGE;               // 128 KiB

// rows rb..rb+3 (first read) and rb+4..rb+7 (second read) of this lane's element: the 8 contraction elements one lane
// feeds to a 32x32x16 MFMA
__device__ __forceinline__ frag8 read_frag(const char* p) {
    const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v*)(p));
    const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v*)(p + 4 * ROWB));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int N>
__device__ __forceinline__ void wait_vmem() {          // until at most N of this wavefront's vector-memory operations are pending
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// The barrier alone: every wavefront has waited for its own loads before it, and the LDS reads still in flight touch
// a stage that nobody writes before the next barrier, so nothing else has to drain here.
__device__ __forceinline__ void stage_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

struct Bf16 {
    static __device__ __forceinline__ acc16 mfma(frag8 a, frag8 b, acc16 c) {
        typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
    }
};
struct F16 {
    static __device__ __forceinline__ acc16 mfma(frag8 a, frag8 b, acc16 c) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
    }
};

// byte offsets of the lane's four A and four B fragments inside a stage (B's include the B tile's offset)
__device__ __forceinline__ void fragment_offsets(int (&offA)[4], int (&offB)[4]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;                            // 2 x 2 wavefronts, each 128 rows x 128 columns of the tile
    // 16-lane group g = lane/16 takes elements 16 (g%2) .. +15 of a 32-element fragment and the row half g/2 of a 16-row
    // half step; lane j of the group addresses row j/4, elements 4 (j%4) .. +3
    const int jj = lane & 15, gg = lane >> 4;
    const int rd_row = (8 * (gg >> 1) + (jj >> 2)) * ROWB + 8 * (jj & 1);
    const int rd_chunk = 2 * (gg & 1) + ((jj & 3) >> 1), rd_swz = jj & 12;
#pragma unroll
    for (int b = 0; b < 4; ++b) offA[b] = rd_row + (((wm * 16 + 4 * b + rd_chunk) ^ rd_swz) << 4);
#pragma unroll
    for (int b = 0; b < 4; ++b) offB[b] = rd_row + (((wn * 16 + 4 * b + rd_chunk) ^ rd_swz) << 4) + TILE_BYTES;
}

// acc += A^T B over `n_steps` >= 1 steps of 32 contraction rows.  a_base / b_base point at the first row's first element
// of the tile's 256 columns in A / B; consecutive rows are a_row_bytes / b_row_bytes apart (at most 128 KiB, 16-byte
// aligned).  From step `alt_from` on the A rows are taken from a_alt_base instead (same geometry; pass n_steps to never
// switch).  Every address touched must be readable: rows 0 .. 32 n_steps - 1, 512 bytes each.
template <typename Mfma>
__device__ __forceinline__ void pipelined(const char* a_base, int64_t a_row_bytes, const char* a_alt_base, int alt_from, const char* b_base,
                                          int64_t b_row_bytes, int n_steps, char* lds, acc16 (&acc)[4][4]) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform, and the compiler knows it
    int offA[4], offB[4];
    fragment_offsets(offA, offB);
    // loads: a step's tiles are 32 loads of two rows each; wavefront w issues loads w, w+4, ...: its first four go to the
    // A tile, the other four to the B tile.  Per load the lane's byte offset from the first row of the step is fixed, and
    // so is the load's place in a stage.
    constexpr int PW = 8;                  // loads of this wavefront per step
    const int lrow = lane >> 5, lpos = lane & 31;
    uint32_t src_off[PW];                  // per lane
    uint32_t dst_off[PW];                  // uniform
#pragma unroll
    for (int q = 0; q < PW; ++q) {
        const int g = wave + 4 * q;                           // 0..15: A tile, 16..31: B tile
        const int op = g >> 4, rp = g & 15;
        const int row = 2 * rp + lrow;
        const int chunk = lpos ^ (4 * (row & 3));
        src_off[q] = (uint32_t)((int64_t)row * (op ? b_row_bytes : a_row_bytes) + 16 * chunk);
        dst_off[q] = (uint32_t)(op * TILE_BYTES + 2 * rp * ROWB);
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds;
    const int64_t a_step = (int64_t)BKS * a_row_bytes, b_step = (int64_t)BKS * b_row_bytes;
    // 16 bytes per lane from global memory straight into LDS at (stage + dst_off) + 16 * lane.  Written as assembly so
    // that the waits stay ours: with the builtin the compiler makes every LDS read wait for all direct loads in flight.
    auto issue_one = [&](const char* base, uint32_t stage_lds, int q) {
        const uint32_t m0v = stage_lds + dst_off[q];
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0v), "v"(src_off[q]), "s"(base) : "m0", "memory");
    };
    // A half step: 16 MFMAs on (af, bfr), the 8 fragments of the next half into (an, bn) from stage address Rn, and one
    // load per quarter (loads lq0 .. lq0+3 of the step whose operand's first row is lbase, into stage lstage).
    auto half = [&](const frag8 (&af)[4], const frag8 (&bfr)[4], frag8 (&an)[4], frag8 (&bn)[4], const char* Rn, const char* lbase,
                    uint32_t lstage, int lq0) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            issue_one(lbase, lstage, lq0 + a);
            // in the order the next half's MFMAs want them
            if (a == 0) { an[0] = read_frag(Rn + offA[0]); bn[0] = read_frag(Rn + offB[0]); }
            if (a == 1) { bn[1] = read_frag(Rn + offB[1]); bn[2] = read_frag(Rn + offB[2]); }
            if (a == 2) { bn[3] = read_frag(Rn + offB[3]); an[1] = read_frag(Rn + offA[1]); }
            if (a == 3) { an[2] = read_frag(Rn + offA[2]); an[3] = read_frag(Rn + offA[3]); }
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[a][b] = Mfma::mfma(af[a], bfr[b], acc[a][b]);
            // one LDS read behind each MFMA instead of a block of reads, then a block of MFMAs
#pragma unroll
            for (int i = 0; i < 4; ++i) { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // The loads of step k are issued during steps k-AHEAD (second half: its A rows) and k-AHEAD+1 (first half: its B
    // rows).  Past the end of the contraction the last step is simply loaded again (into a stage nobody reads any more) and
    // the fragments read for the "next" half are not used: every step then runs the same instructions with the same number
    // of loads in flight, the loop needs no special first or last iterations, and the wait counts are constants.
    constexpr int AHEAD = NSTAGE - 1;
    const int last = n_steps - 1;
    auto a_of = [&](int k) { const int kk = k < last ? k : last; return (kk >= alt_from ? a_alt_base : a_base) + (int64_t)kk * a_step; };
    auto b_of = [&](int k) { return b_base + (int64_t)(k < last ? k : last) * b_step; };
    for (int k = 0; k < AHEAD - 1; ++k) {
#pragma unroll
        for (int q = 0; q < PW / 2; ++q) issue_one(a_of(k), lds_base + k * STAGE, q);
#pragma unroll
        for (int q = PW / 2; q < PW; ++q) issue_one(b_of(k), lds_base + k * STAGE, q);
    }
#pragma unroll
    for (int q = 0; q < PW / 2; ++q) issue_one(a_of(AHEAD - 1), lds_base + (AHEAD - 1) * STAGE, q);
    wait_vmem<(AHEAD - 2) * PW + PW / 2>();                    // step 0 has landed
    stage_barrier();
    frag8 a0[4], b0[4], a1[4], b1[4];
    a0[0] = read_frag(lds + offA[0]);
#pragma unroll
    for (int b = 0; b < 4; ++b) b0[b] = read_frag(lds + offB[b]);
#pragma unroll
    for (int b = 1; b < 4; ++b) a0[b] = read_frag(lds + offA[b]);
    int slot = 0;                                              // stage of the current step
    for (int step = 0; step < n_steps; ++step) {
        const char* At = lds + slot * STAGE;
        int s1 = slot + AHEAD - 1; if (s1 >= NSTAGE) s1 -= NSTAGE;
        // first half: rows 0..15; fragments of rows 16..31; the B rows of step+AHEAD-1
        half(a0, b0, a1, b1, At + 16 * ROWB, b_of(step + AHEAD - 1), lds_base + s1 * STAGE, PW / 2);
        wait_vmem<(AHEAD - 2) * PW>();                         // step+1 has landed (each wavefront waits for its own loads)
        stage_barrier();                                       // ... everybody's; and the stage of step-1 is free
        int s2 = slot + AHEAD; if (s2 >= NSTAGE) s2 -= NSTAGE;
        int sn = slot + 1; if (sn >= NSTAGE) sn -= NSTAGE;
        // second half: rows 16..31; fragments of the next step's rows 0..15; the A rows of step+AHEAD
        half(a1, b1, a0, b0, lds + sn * STAGE, a_of(step + AHEAD), lds_base + s2 * STAGE, 0);
        slot = sn;
    }
    wait_vmem<0>();            // nothing may still be on its way into LDS when the workgroup ends
}

}  // namespace tile256
}  // namespace cdq
