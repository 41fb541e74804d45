/* ws_oracle.c -- CPU oracle for the weight-stationary matrix-multiply recurrence.
 *
 * TEST INFRASTRUCTURE.  This file is the slow, literal reference that the GPU
 * library is checked against.  Nothing in the product path may include, link or
 * call it; it shares no code, header, table or helper with the HIP sources.
 *
 * What it simulates (paper, section "Space-time Mappings of Dataflow
 * Recurrences", weight-stationary program, and the figure of nine per-cell
 * programs): an M x K grid of cells; cell (i,k) latches A_ik once; for every
 * time step j the north row reads column j of B from memory, each cell copies
 * the B value of its northern neighbour, adds W*B to the partial sum arriving
 * from its western neighbour (0 at the west boundary), passes B south and the
 * partial sum east, and the east column writes C_ij.
 *
 * Three forms, bit-identical to one another by construction of the method:
 *   ws_cells_*      sequential literal grid, nine programs + degenerate grids
 *   ws_wavefront_*  clocked grid with unit-latency links, checks t = i+j+k
 *   ws_rowchain_*   the same k-ordered chain per (i,j) without the grid state
 *
 * Two arithmetic modes:
 *   i8   A,B int8; partial sums int32 with two's-complement wrap
 *   bf16 A,B bfloat16 (passed as uint16 bit patterns); widened exactly to
 *        fp32; product and sum in fp32, round-to-nearest-even, one rounding
 *        per add (the 8-bit x 8-bit significand product is exact in fp32
 *        barring under/overflow, so fused and unfused multiply-add agree);
 *        the chain starts from +0.0f.  Build with -ffp-contract=off, no fast-math.
 *
 * Readings where the paper is loose: loops are written from 1 there, indices
 * are 0-based here; cell k = 0 is a real cell that computes 0 + W*B (as its
 * per-cell program shows), the zero is a virtual feeder; the "forward B" line
 * of the weight-stationary program carries a C subscript on its target, which
 * is a slip for B; the (i,0) box ends in an emit, which is a slip for the east
 * forward; the caption's "time coordinate k" is j.  Summation order for floats
 * is strictly k = 0..K-1, as the chain implies.
 *
 * Parity pins (tests/test_oracle_pins.py): library int64 / fp64 matmul on
 * small shapes, identity weights, rank-1 outer products, all-ones, one-hot
 * probes, the sum identity, the tick count M+K+N-2 with no mis-timed operand.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------- int8 -> int32 ---------------- */
static inline int32_t mac_i8(int32_t c, int8_t w, int8_t b)
{
    int32_t p = (int32_t)w * (int32_t)b;
    return (int32_t)((uint32_t)c + (uint32_t)p);   /* wraps mod 2^32 */
}
#define ELEM int8_t
#define ACC int32_t
#define ACC_ZERO 0
#define MAC(c, w, b) mac_i8((c), (w), (b))
#define FN(name) name##_i8
#include "ws_grid.inc"
#undef ELEM
#undef ACC
#undef ACC_ZERO
#undef MAC
#undef FN

/* ---------------- bf16 -> fp32 ---------------- */
static inline float widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}
static inline float mac_bf16(float c, uint16_t w, uint16_t b)
{
    float p = widen_bf16(w) * widen_bf16(b);   /* exact in fp32 for in-range data */
    return c + p;                              /* one rounding, nearest even      */
}
#define ELEM uint16_t
#define ACC float
#define ACC_ZERO 0.0f
#define MAC(c, w, b) mac_bf16((c), (w), (b))
#define FN(name) name##_bf16
#include "ws_grid.inc"
#undef ELEM
#undef ACC
#undef ACC_ZERO
#undef MAC
#undef FN

int ws_oracle_threads(void);
#ifdef _OPENMP
#include <omp.h>
int ws_oracle_threads(void) { return omp_get_max_threads(); }
#else
int ws_oracle_threads(void) { return 1; }
#endif
