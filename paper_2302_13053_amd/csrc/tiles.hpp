// Pieces shared by the MFMA kernels (dense transform and weight gradient).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileK = 16;    // K extent of one LDS tile

// Four consecutive floats starting at base[off], fetched without a branch: an
// element that is not wanted (or would be out of range) is fetched from base[0]
// instead; zero4 later replaces it by zero.  Keeping the replacement out of the
// load lets all loads of a K step stay in flight behind the MFMAs of the
// previous step.
//   VEC: the four are one aligned 16-byte load and are wanted all or none
template <bool VEC>
__device__ __forceinline__ void load4(const float* __restrict__ base, int64_t off, int wanted, float (&r)[4])
{
    if constexpr (VEC) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(base + (wanted >= 4 ? off : 0));
        r[0] = t.x; r[1] = t.y; r[2] = t.z; r[3] = t.w;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = base[q < wanted ? off + q : 0];
    }
}

template <bool VEC>
__device__ __forceinline__ void zero4(int wanted, float (&r)[4])
{
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = (VEC ? wanted >= 4 : q < wanted) ? r[q] : 0.0f;
}


// ---------------------------------------------------------------------------
// Software-pipelined K loop of one workgroup tile (four waves, fp32 32x32x2 MFMA).
//
// One wave keeps a matrix core busy only if nothing else in its instruction
// stream takes longer than one MFMA (64 cycles).  The loop therefore cuts all
// staging work into pieces of about that size and places them between the MFMAs
// of the wave that does them; sched_barrier pins the order.  Per K step (kTileK
// columns = 8 k-steps of 2):
//   after the first MFMA of every k-step: LDS reads of the next k-step's operands
//   after the second MFMA of k-steps 0..2: put(buf ^ 1, 0..2), one third each of
//       "write tile t+1 from the staging registers to the other LDS buffer"
//   after the second MFMA of k-steps 3, 4: fetch(t + 2, 0 / 1), the two halves of
//       "load tile t+2 into the staging registers" (so a global load has a whole K
//       step of MFMAs to arrive)
//   between k-steps 6 and 7 (operands of 7 already in registers): the one barrier,
//       then the reads of the next tile's first operands behind k-step 7's MFMAs.
// Contract on entry: tile 0 is in LDS buffer 0 and a barrier has passed; tile 1
// (if nk > 1) is in the caller's staging registers.  LDS tiles are k-major:
// As[buf][k][row of the workgroup tile], Bs[buf][k][column]; a0 / b0 are the first
// row / column of this wave's TM x TN block of 32 x 32 accumulators.  last_steps:
// k-steps of the last tile that hold data (a K extent that is not a multiple of
// kTileK leaves the others zero-filled; they are skipped).
// ---------------------------------------------------------------------------
#define RETEXO_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int TM, int TN, int LDA, int LDB, class Put, class Fetch>
__device__ __forceinline__ void mfma_k_loop(f32x16 (&acc)[TM][TN], const float (*As)[kTileK][LDA],
                                            const float (*Bs)[kTileK][LDB], int nk, int a0, int b0, int lane,
                                            Put&& put, Fetch&& fetch, int last_steps = kTileK / 2)
{
    constexpr int NSTEP = kTileK / 2;
    static_assert(NSTEP == 8, "the schedule below is written for 8 k-steps");
    const int lrow = lane & 31, lk = lane >> 5;
    float af[2][TM], bf[2][TN];
    auto frag = [&](int buf, int s, int slot) {       // operands of k-step s -> register set slot
#pragma unroll
        for (int i = 0; i < TM; ++i) af[slot][i] = As[buf][2 * s + lk][a0 + i * 32 + lrow];
#pragma unroll
        for (int j = 0; j < TN; ++j) bf[slot][j] = Bs[buf][2 * s + lk][b0 + j * 32 + lrow];
    };
    frag(0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < nk;        // the staging registers hold tile kt + 1
        const bool more2 = kt + 2 < nk;
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            if (!more && s >= last_steps) break;   // the rest of a partial last tile is zeros: adds nothing, changes no bit
            const int cur = s & 1;
            int q = 0;                        // MFMAs issued in this k-step
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][i], bf[cur][j], acc[i][j], 0, 0, 0);
                    RETEXO_SCHED_FENCE();
                    if (q == 0) {
                        if (s + 1 < NSTEP) frag(buf, s + 1, cur ^ 1);
                        RETEXO_SCHED_FENCE();
                    }
                    if (q == (TM * TN > 1 ? 1 : 0)) {
                        if (s <= 2 && more) put(buf ^ 1, s);
                        if (s == 3 && more2) fetch(kt + 2, 0);
                        if (s == 4 && more2) fetch(kt + 2, 1);
                        RETEXO_SCHED_FENCE();
                    }
                    ++q;
                }
            }
            if (s == NSTEP - 2) {
                // every wave has read its last operands of this tile and written its share of the next one;
                // the barrier waits for LDS traffic only, global loads stay in flight across it
                __syncthreads();
                RETEXO_SCHED_FENCE();
                if (more) frag(buf ^ 1, 0, 0);
                RETEXO_SCHED_FENCE();
            }
        }
    }
}
